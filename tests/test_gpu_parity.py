"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Error measure per tensor: max |gpu - oracle| / max |oracle|.
Gates: fp32 path <= 1e-4; bf16 path <= 2e-2 on features / logits / depth and >= 0.99 agreement
of the segmentation and detection class maps (the oracle's argmax is taken on its fp64 scores).
Depth maps: the same measure; both it and the error relative to the map before its final ReLU are printed,
and a map that the ReLU clips (its maximum below a quarter of the pre-ReLU magnitude: with random weights
that happens) is held to the second form instead (helpers.depth_gate).
"""
import numpy as np
import pytest
import torch

import paper_2508_11584_amd as vpe
import vpe_inputs as vi
from helpers import depth_errs, depth_gate, make_engine, relerr
from oracle import model, ops

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def run_gpu(eng, images, n_heads):
    """One frame through encode + all heads; returns (features [4 x (B,N,D)], head outputs)."""
    img = torch.from_numpy(images).cuda().contiguous()
    fh = eng.encode(img)
    for h in range(n_heads):
        assert eng.run_head(h, fh) == 0
    eng.sync()
    feats = [eng.feat_view(fh, k).float().cpu().numpy() for k in range(4)]
    return fh, feats


def regret(scores, ref_cls, got_cls):
    """max over positions of oracle score of the oracle's class minus oracle score of the GPU's class."""
    s = np.asarray(scores)
    a = np.take_along_axis(s, np.asarray(ref_cls, dtype=np.int64)[None], 0)[0]
    b = np.take_along_axis(s, np.asarray(got_cls, dtype=np.int64)[None], 0)[0]
    return float(np.max(a - b))


def head_outputs(eng, kinds):
    """Host copies of every output of every head: [[output 0, output 1 (class map, if the head has one)], ...]."""
    return [[eng.head_output(hi, which).cpu().numpy().copy() for which in range(2 if kind in ("seg", "det") else 1)]
            for hi, kind in enumerate(kinds)]


def compare_with_oracle(spec, w, hw, kinds, images, feats, outs, batch_check=None):
    """Runs the oracle on the checked batch elements and applies the gates.  feats: four [B][N][D] host arrays;
    outs: as head_outputs returns them."""
    tol = TOL[spec.dtype]
    report = {}
    for b in (range(spec.batch) if batch_check is None else batch_check):
        ofe = model.encode_image(spec, w, images[b])
        for k in range(4):
            report[f"b{b}.feat{k}"] = relerr(feats[k][b], ofe[k])
        for hi, kind in enumerate(kinds):
            if kind == "seg":
                o = model.seg_head(spec, hw[hi], ofe)
                logits = outs[hi][0][b]                                       # [gh][gw][C]
                report[f"b{b}.h{hi}.seg.logits"] = relerr(logits.transpose(2, 0, 1), o["logits"])
                cm = outs[hi][1][b]
                report[f"b{b}.h{hi}.seg.agree"] = float(np.mean(cm == o["classmap"]))
                # a differing pixel is valid only if it is a near-tie: picking class g over the oracle's o
                # implies oracle[o] - oracle[g] <= 2 max |logit error| (interpolation is a convex combination)
                up = ops.bilinear(o["logits"], spec.img_h, spec.img_w)
                err = np.max(np.abs(logits.transpose(2, 0, 1) - o["logits"]))
                report[f"b{b}.h{hi}.seg.regret_ok"] = bool(regret(up, o["classmap"], cm) <= 2 * err + 1e-6)
            elif kind == "det":
                o = model.det_head(spec, hw[hi], ofe)
                out = outs[hi][0][b]                                          # [gh][gw][K+4]
                K = spec.det_classes
                report[f"b{b}.h{hi}.det.logits"] = relerr(out[..., :K].transpose(2, 0, 1), o["logits"])
                report[f"b{b}.h{hi}.det.box"] = relerr(out[..., K:].transpose(2, 0, 1), o["box"])
                cm = outs[hi][1][b]
                report[f"b{b}.h{hi}.det.agree"] = float(np.mean(cm == o["classmap"]))
                err = np.max(np.abs(out[..., :K].transpose(2, 0, 1) - o["logits"]))
                report[f"b{b}.h{hi}.det.regret_ok"] = bool(regret(o["logits"], o["classmap"], cm) <= 2 * err + 1e-6)
            else:
                o = (model.dpt_head if kind == "dpt" else model.depth_head)(spec, hw[hi], ofe)
                d = outs[hi][0][b]
                assert d.min() >= 0.0 and d.shape == (spec.img_h, spec.img_w)
                errs = depth_errs(d, o)
                report.update({f"b{b}.h{hi}.{kind}.{k}": v for k, v in errs.items()})
                report[f"b{b}.h{hi}.{kind}.gate_ok"] = depth_gate(errs, tol)
    print(spec.name, {k: (v if isinstance(v, bool) else round(v, 6) if v < 0.5 else round(v, 4))
                      for k, v in report.items()}, flush=True)
    # class maps: >= 0.99 agreement on maps large enough for the fraction to mean something (one cell of a
    # 165-cell map is already 0.6 %); on small maps >= 0.95, and every disagreement must be a near-tie
    cells = spec.patches
    for k, v in report.items():
        if k.endswith("regret_ok") or k.endswith("gate_ok"):
            assert v, (k, report)
        elif ".depth." in k or ".dpt." in k:
            pass                                # both normalisations are printed; gate_ok carries the decision
        elif k.endswith("agree"):
            floor = 0.999 if spec.dtype == "f32" else 0.99 if (cells >= 1000 or "seg" in k) else 0.95
            assert v >= floor, (k, v)
        else:
            assert v <= tol, (k, v)
    return report


def check_all(spec, seed, img_seed, kinds=("seg", "depth", "det"), flags=0, batch_check=None, lead_frames=0,
              weights_edit=None, on_device=None, **engine_kw):
    """One frame through the engine, then the oracle on the same inputs (the engine is closed before the oracle
    starts: the GPU is not held while the CPU works).  on_device(eng, images, fh, feats, outs) may add device-side
    checks while the engine is alive."""
    if weights_edit is not None:               # same generator, then an in-place change both sides will see
        engine_kw["weights"] = vi.make_backbone_weights(spec, seed)
        weights_edit(engine_kw["weights"])
    eng, w, hw = make_engine(spec, seed, kinds=kinds, flags=flags, **engine_kw)
    images = vi.make_batch(spec, img_seed)
    # optional lead-in: other frames pushed through encode + heads with no host synchronisation, so that the
    # checked frame runs in a filled pipeline (its slot, lane and graph are not the first ones)
    lead = [torch.from_numpy(vi.make_batch(spec, img_seed + 100 + i)).cuda() for i in range(min(lead_frames, 2))]
    for i in range(lead_frames):
        lf = eng.encode(lead[i % len(lead)])
        for h in range(len(kinds)):
            eng.run_head(h, lf)
    fh, feats = run_gpu(eng, images, len(kinds))
    outs = head_outputs(eng, kinds)
    if on_device is not None:
        on_device(eng, images, fh, feats, outs)
    eng.close()
    return compare_with_oracle(spec, w, hw, kinds, images, feats, outs, batch_check)


MEDIUM = dict(dim=128, depth=4, heads=2, mlp_hidden=256, img_h=154, img_w=210, taps=(1, 2, 3, 4), head_ch=64)


def test_medium_fp32_all_heads():
    # 11 x 15 = 165 patches, N = 166: more than one 128-row tile plus a ragged tail
    check_all(vi.ModelSpec("medium_f32", dtype="f32", **MEDIUM), 101, 201)


def test_medium_bf16_all_heads():
    check_all(vi.ModelSpec("medium_bf16", dtype="bf16", **MEDIUM), 102, 202)


def test_swiglu_registers_batch_bf16():
    spec = vi.ModelSpec("swiglu_b3", dtype="bf16", **{**MEDIUM, "mlp_kind": vi.MLP_SWIGLU, "registers": 4, "batch": 3,
                                                       "img_h": 70, "img_w": 98, "seg_classes": 150})
    check_all(spec, 103, 203)


def test_swiglu_registers_batch_fp32():
    spec = vi.ModelSpec("swiglu_b2_f32", dtype="f32", **{**MEDIUM, "mlp_kind": vi.MLP_SWIGLU, "registers": 4,
                                                           "batch": 2, "img_h": 70, "img_w": 98})
    check_all(spec, 104, 204)


def test_single_patch_image():
    # degenerate grid: 1 x 1 patches, N = 2, every bilinear resize clamps everywhere
    for dt in ("f32", "bf16"):
        check_all(vi.ModelSpec("one_patch_" + dt, dtype=dt, **{**MEDIUM, "img_h": 14, "img_w": 14}), 105, 205)


def test_one_row_of_patches():
    check_all(vi.ModelSpec("strip", dtype="bf16", **{**MEDIUM, "img_h": 14, "img_w": 14 * 67}), 106, 206)


def test_widest_supported_model():
    # the limits the library accepts: width 2048 (32 heads: 32 statistics groups per row, LayerNorm rows of 16
    # float2 per lane), 64 register tokens, 255 segmentation classes, 1024 head channels; four blocks, a 2 x 3 grid
    spec = vi.ModelSpec("widest", dtype="bf16", dim=2048, depth=4, heads=32, mlp_hidden=2048, registers=64, img_h=28,
                        img_w=42, taps=(1, 2, 3, 4), seg_classes=255, head_ch=1024)
    check_all(spec, 107, 207)


def test_cfg1_vits_fp32_224_seg():
    # benchmark configuration 1: ViT-S/14 fp32, 224 x 224, linear seg head; gate 1e-4
    spec = vi.CONFIGS["cfg1"]
    check_all(spec, *vi.SEEDS["cfg1"], kinds=("seg",))


def test_cfg2_vits_bf16_476x630_three_heads():
    # benchmark configuration 2 (the headline one), whole, all three heads, as bench.py runs it
    spec = vi.CONFIGS["cfg2"]
    check_all(spec, *vi.SEEDS["cfg2"], flags=vpe.VPE_FLAG_GRAPHS)


def test_residual_stream_with_a_large_common_offset():
    # every token carries a level of +30 (patch bias and CLS) on top of deviations of order 1, and keeps it through
    # all blocks: the in-GEMM LayerNorm statistics must come from differences, not from raw sums of squares
    # (E[x^2] - mean^2 in fp32 would lose four digits here and miss the 1e-4 gate)
    def lift(w, by):
        w["patch_b"] += np.float32(by)
        w["cls"] += np.float32(by)
    check_all(vi.ModelSpec("offset30_f32", dtype="f32", **MEDIUM), 104, 204, weights_edit=lambda w: lift(w, 30.0))
    # the bf16 engine multiplies a 16-bit copy of the stream itself, stored relative to each row's level (the
    # mean the previous LayerNorm saw, or bias + positional row for a fresh frame): the same lift must not
    # cost it its ordinary gate either
    check_all(vi.ModelSpec("offset30_bf16", dtype="bf16", **MEDIUM), 105, 205, weights_edit=lambda w: lift(w, 30.0))


def test_cfg2_in_the_pipelined_configuration_the_benchmark_times():
    # as bench.py launches it: three encoder lanes, a ring of four slots, HIP graphs, frames in flight
    spec = vi.CONFIGS["cfg2"]
    check_all(spec, *vi.SEEDS["cfg2"], flags=vpe.VPE_FLAG_GRAPHS, lead_frames=6, ring_slots=4, encoder_lanes=3)


@pytest.mark.parametrize("tile", ["384", "256", "128", "65", "64", "4"])
def test_direct_to_lds_gemm_variant(tile, monkeypatch):
    # each direct-to-LDS GEMM shape (384 x 256, 256 x 256, 256 x 128, 64 x 128, 64 x 64 tiles) and the split-k 64 x 64
    # shape ("4": two wave groups over halves of the k range, odd and even k-tile counts), forced for every GEMM of the model,
    # through every epilogue: folded LayerNorm + QKV with transposed values, LayerScale residual with row
    # statistics, GELU and SwiGLU, patch embedding, 1x1 and 3x3 convolutions, the fused 1-channel projection
    monkeypatch.setenv("VPE_GEMM_TILE", tile)
    check_all(vi.ModelSpec("medium_bf16_tile" + tile, dtype="bf16", **MEDIUM), 102, 202)
    spec = vi.ModelSpec("swiglu_tile" + tile, dtype="bf16", **{**MEDIUM, "mlp_kind": vi.MLP_SWIGLU, "registers": 4,
                                                                "batch": 3, "img_h": 70, "img_w": 98})
    check_all(spec, 103, 203)


@pytest.mark.parametrize("shape", ["1", "2"])
def test_strip_convolution_kernel(shape, monkeypatch):
    # the 3x3 convolution that forms its nine taps from one input strip in LDS, in both of its tile shapes (1: 384 x 256,
    # 2: 768 x 128), forced for every convolution it can take (whole tiles of output channels): detection towers reading
    # token rows of two images with register tokens in between, the depth head's four fusion stages on 11x15 ... 88x120
    # grids (tiles that span several image rows, both images and the end of the tensor; taps masked at every edge), the
    # last with the 1-channel projection
    monkeypatch.setenv("VPE_GEMM_TILE", "9")
    monkeypatch.setenv("VPE_STRIP_SHAPE", shape)
    spec = vi.ModelSpec("strip_conv", dtype="bf16", **{**MEDIUM, "head_ch": 256, "batch": 2, "registers": 4})
    check_all(spec, 108, 208)
    # one row of patches (every pixel on the top and bottom edge) and a single patch
    check_all(vi.ModelSpec("strip_conv_row", dtype="bf16", **{**MEDIUM, "head_ch": 256, "img_h": 14, "img_w": 14 * 9}), 109, 209)
    check_all(vi.ModelSpec("strip_conv_1x1", dtype="bf16", **{**MEDIUM, "head_ch": 256, "img_h": 14, "img_w": 14}), 110, 210)


# ---------------------------------------------------------------- full DPT head
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dpt_head_small_grids_odd_and_even(dtype):
    # 11 x 15 patches: the deepest level is 6 x 8 (odd grid halved with padding), resizes 6x8 -> 11x15 are not x2
    check_all(vi.ModelSpec("dpt_odd_" + dtype, dtype=dtype, **MEDIUM), 131, 231, kinds=("dpt",))
    # two images, registers, an even grid, together with the other heads (shared features)
    spec = vi.ModelSpec("dpt_even_" + dtype, dtype=dtype, **{**MEDIUM, "registers": 4, "batch": 2, "img_h": 112, "img_w": 140})
    check_all(spec, 132, 232, kinds=("seg", "dpt", "det"))


def test_dpt_head_degenerate_grids():
    # one patch (every level at least 1 x 1, resizes from a single sample) and one row of patches
    for dt in ("f32", "bf16"):
        check_all(vi.ModelSpec("dpt_one_patch_" + dt, dtype=dt, **{**MEDIUM, "img_h": 14, "img_w": 14}), 135, 235, kinds=("dpt",))
    check_all(vi.ModelSpec("dpt_strip", dtype="bf16", **{**MEDIUM, "img_h": 14, "img_w": 14 * 23}), 136, 236, kinds=("dpt",))


def test_dpt_head_wider_and_under_graph_replay():
    spec = vi.ModelSpec("dpt_wide", dtype="bf16", **{**MEDIUM, "head_ch": 128, "img_h": 98, "img_w": 126})
    check_all(spec, 133, 233, kinds=("dpt", "depth"), flags=vpe.VPE_FLAG_GRAPHS, lead_frames=3, ring_slots=2)


def test_dpt_head_at_its_widest():
    # width 256 (the DepthAnythingV2-large head shape): reassembled widths 192 .. 1536, no channel padding anywhere
    spec = vi.ModelSpec("dpt_256", dtype="bf16", **{**MEDIUM, "head_ch": 256, "img_h": 70, "img_w": 98, "batch": 2})
    check_all(spec, 134, 234, kinds=("dpt",))


def test_dpt_head_at_the_benchmark_size():
    # ViT-S/14 at 476 x 630 with the DepthAnythingV2-small head shape (width 64, reassembled widths 48 .. 384):
    # levels 136x180, 68x90, 34x45, 17x23; output convolutions on 272x360 and 476x630
    spec = vi.with_(vi.CONFIGS["cfg2"], head_ch=64, name="cfg2_dpt")
    check_all(spec, *vi.SEEDS["cfg2"], kinds=("dpt",), flags=vpe.VPE_FLAG_GRAPHS, lead_frames=2, ring_slots=2)


# ---------------------------------------------------------------- camera-frame transform
@pytest.mark.parametrize("src,dst,batch", [((1080, 1920), (476, 630), 1),      # the paper's camera frames -> cfg 2
                                           ((1080, 1920), (518, 518), 2),      # -> cfgs 3-5, two views
                                           ((37, 53), (98, 154), 1),           # enlargement, odd sizes
                                           ((224, 224), (224, 224), 1),        # same size: conversion only
                                           ((1, 1), (14, 14), 1),              # degenerate source
                                           ((300, 7), (14, 700), 3)])          # ragged: shrink one axis, stretch the other
def test_preprocess_u8_matches_the_oracle(src, dst, batch):
    frames = np.stack([vi.make_camera_frame(src[0], src[1], 40 + b) for b in range(batch)])
    dev = torch.from_numpy(frames).cuda()
    out = torch.full((batch, 3, dst[0], dst[1]), float("nan"), dtype=torch.float32, device="cuda")
    vpe.preprocess_u8(dev, out, vi.CAMERA_MEAN, vi.CAMERA_STD)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for b in range(batch):
        ref = model.preprocess_u8(frames[b], dst[0], dst[1], vi.CAMERA_MEAN, vi.CAMERA_STD)
        err = float(np.max(np.abs(got[b] - ref)) / np.max(np.abs(ref)))
        print("preprocess", src, dst, b, err, flush=True)
        assert err <= 2e-6                      # exact tap positions; fp32 weights, blend, one scale and one shift


def test_preprocessed_camera_frame_runs_through_the_engine():
    # the transform's output is a valid engine input: same features as feeding the oracle's transform
    spec = vi.small_spec()
    eng, w, _ = make_engine(spec, 7, kinds=("seg",))
    frame = vi.make_camera_frame(90, 160, 77)
    dev = torch.from_numpy(frame[None]).cuda()
    img = torch.empty((1, 3, spec.img_h, spec.img_w), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()                   # the frame upload; from here on the engine's own stream orders the work
    vpe.preprocess_u8(dev, img, vi.CAMERA_MEAN, vi.CAMERA_STD, stream=eng.next_encode_stream())
    fh = eng.encode(img)
    eng.sync()
    got = eng.feat_view(fh, 3).float().cpu().numpy()[0]
    ref_img = model.preprocess_u8(frame, spec.img_h, spec.img_w, vi.CAMERA_MEAN, vi.CAMERA_STD)
    feats = model.encode_image(spec, w, ref_img.astype(np.float32))
    assert relerr(got, feats[3]) <= (1e-4 if spec.dtype == "f32" else 2e-2)
    eng.close()


# ---------------------------------------------------------------- several heads of one kind (paper, Sec. "Parallel
# vs. Sequential Processing" and "Single Backbone vs. Independent Models": k heads of one kind on one backbone)
def test_four_depth_heads_on_one_backbone_each_match_the_oracle():
    # four DPT-lite heads with different weights share the feature slot; more heads than head streams, so two
    # share a stream.  Every replica is compared with the oracle run on its own weights.
    spec = vi.CONFIGS["cfg2"]
    rep = check_all(spec, *vi.SEEDS["cfg2"], kinds=("depth",) * 4)
    assert len({round(rep[f"b0.h{h}.depth.pre_relu"], 9) for h in range(4)}) > 1      # different heads, not copies


def test_eight_detection_heads_in_the_pipelined_configuration():
    spec = vi.CONFIGS["cfg2"]
    check_all(spec, *vi.SEEDS["cfg2"], kinds=("det",) * 8, flags=vpe.VPE_FLAG_GRAPHS, lead_frames=5, ring_slots=4,
              encoder_lanes=3)


# ---------------------------------------------------------------- attention far from uniform
SHARP = dict(dim=128, depth=4, heads=2, mlp_hidden=256, img_h=14 * 18, img_w=14 * 20, taps=(1, 2, 3, 4), head_ch=64)


def _sharpen(scale):
    def edit(w):
        # queries and keys (the first two thirds of the fused projection) scaled up: scores grow by scale^2, the
        # softmax concentrates on a few keys per query, and which keys differs from one key tile to the next
        for name in list(w):
            if name.endswith("qkv_w"):
                w[name][:, : 2 * w[name].shape[1] // 3] *= np.float32(scale)
            elif name.endswith("qkv_b"):
                w[name][: 2 * w[name].shape[0] // 3] *= np.float32(scale)
    return edit


@pytest.mark.parametrize("dtype,variant,scale", [("bf16", "124", 16.0), ("bf16", "224", 16.0), ("bf16", "141", 16.0),
                                                 ("bf16", "114", 16.0), ("bf16", "214", 16.0), ("bf16", "122", 16.0),
                                                 ("bf16", "", 16.0),
                                                 ("f32", "114", 32.0), ("f32", "141", 32.0)])
def test_attention_with_peaked_softmax(dtype, variant, scale, monkeypatch):
    # 361 tokens = six key tiles of 64 (the last with 41 keys): with four key waves two of them own two tiles.
    # With the benchmark's weights every score lies within a fraction of a unit of the others, so the running
    # maximum never grows after the first tile and the partial results of the key waves are nearly equal; here
    # scores spread over tens of units, so rescaling on a growing maximum, the merge of partials taken against
    # different references and the masked tail all carry weight.
    if variant:
        monkeypatch.setenv("VPE_ATTN_VARIANT", variant)
    spec = vi.ModelSpec(f"sharp_{dtype}_{variant or 'auto'}", dtype=dtype, **SHARP)
    rep = check_all(spec, 141, 241, kinds=("seg",), weights_edit=_sharpen(scale))
    assert rep["b0.feat3"] > 0.0
