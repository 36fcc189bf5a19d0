"""The encoder and the three task heads, written out with the fp64 oracle operators.

TEST INFRASTRUCTURE ONLY (see the package docstring).

What is computed follows the paper's Sec. "Example implementation": a DINOv2-style
ViT/14 encoder configured to output its final features plus three evenly spaced
intermediate layers, read by a DPT-style depth head, a linear segmentation head and
a detection head.  The paper prints no formulas, so every step is the standard
definition of the named layer; choices the paper leaves open are stated where made.

`spec` is any object with the attributes of `vpe_inputs.ModelSpec`; `w` is a dict of
arrays named as in `vpe_inputs.backbone_layout` / `head_layout`.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import ops

MLP_SWIGLU = 1


def preprocess_u8(frame, H: int, W: int, mean, std) -> np.ndarray:
    """Camera-frame transform (paper, Sec. "Transforms": type conversion, resizing, normalisation).

    frame [Hs][Ws][3] uint8 interleaved RGB -> [3][H][W]: each channel scaled to 0..1, resized bilinearly
    (half-pixel centres, no antialiasing filter; nothing is rounded back to integers), then (v - mean_c) / std_c.
    """
    f = np.asarray(frame)
    assert f.dtype == np.uint8 and f.ndim == 3 and f.shape[2] == 3
    planes = np.ascontiguousarray(f.transpose(2, 0, 1)).astype(np.float64) / 255.0
    r = ops.bilinear(planes, H, W)
    m = np.asarray(mean, dtype=np.float64).reshape(3, 1, 1)
    s = np.asarray(std, dtype=np.float64).reshape(3, 1, 1)
    return (r - m) / s


def tokens_from_image(spec, w, img) -> np.ndarray:
    """x0 [N][D]: CLS + pos[0]; registers (no positional term); patch p + pos[1+p].

    Patch embedding is the 14x14 stride-14 convolution; the positional table has
    1+P rows (generated at the grid size, never interpolated); register tokens sit
    between CLS and the patches and receive no positional embedding.
    """
    D, R = spec.dim, spec.registers
    t = ops.patch_embed(img, w["patch_w"], w["patch_b"], 14)
    pos = np.asarray(w["pos"], dtype=np.float64)
    x = np.empty((spec.tokens, D))
    x[0] = np.asarray(w["cls"], dtype=np.float64) + pos[0]
    if R:
        x[1:1 + R] = np.asarray(w["reg"], dtype=np.float64)
    x[1 + R:] = t + pos[1:]
    return x


def block(spec, w, l: int, x: np.ndarray) -> np.ndarray:
    """One pre-LN transformer block with LayerScale on both residual branches."""
    p = f"blk{l}."
    u = ops.layernorm(x, w[p + "ln1_g"], w[p + "ln1_b"], spec.ln_eps)
    qkv = ops.linear(u, w[p + "qkv_w"], w[p + "qkv_b"])
    a = ops.attention(qkv, spec.heads, spec.head_dim)
    x = ops.scale_residual(x, ops.linear(a, w[p + "proj_w"], w[p + "proj_b"]), w[p + "ls1"])
    u = ops.layernorm(x, w[p + "ln2_g"], w[p + "ln2_b"], spec.ln_eps)
    hdn = ops.linear(u, w[p + "fc1_w"], w[p + "fc1_b"])
    hdn = ops.swiglu(hdn) if spec.mlp_kind == MLP_SWIGLU else ops.gelu(hdn)
    x = ops.scale_residual(x, ops.linear(hdn, w[p + "fc2_w"], w[p + "fc2_b"]), w[p + "ls2"])
    return x


def encode_image(spec, w, img, return_blocks: bool = False):
    """Encoder forward for one image [3][H][W].

    Returns the four feature maps F_0..F_3, each [N][D]: the shared final LayerNorm
    applied to the residual stream after the blocks listed in spec.taps (1-based);
    F_3 (after the last block) is "the final tokens".  With return_blocks also returns
    the raw residual stream after every block (x0 first).
    """
    x = tokens_from_image(spec, w, img)
    feats: List[np.ndarray] = []
    stream = [x.copy()]
    for l in range(spec.depth):
        x = block(spec, w, l, x)
        if return_blocks:
            stream.append(x.copy())
        if (l + 1) in spec.taps:
            feats.append(ops.layernorm(x, w["norm_g"], w["norm_b"], spec.ln_eps))
    assert len(feats) == 4 and spec.taps[3] == spec.depth
    return (feats, stream) if return_blocks else feats


def encode(spec, w, images) -> List[np.ndarray]:
    """Batched encoder: images [B][3][H][W] -> four arrays [B][N][D]."""
    per = [encode_image(spec, w, im) for im in images]
    return [np.stack([per[b][k] for b in range(len(per))]) for k in range(4)]


def _grid(spec, feat) -> np.ndarray:
    """Patch rows of one feature map [N][D] as a channels-first grid [D][gh][gw]."""
    g = np.asarray(feat, dtype=np.float64)[1 + spec.registers:]
    return np.ascontiguousarray(g.reshape(spec.gh, spec.gw, spec.dim).transpose(2, 0, 1))


def _decide(z: np.ndarray) -> np.ndarray:
    """Channel argmax of the fp64 scores (ties -> lowest index)."""
    return ops.argmax_channels(np.asarray(z, dtype=np.float64))


def seg_head(spec, hw, feats) -> Dict[str, np.ndarray]:
    """Linear segmentation head on one image's features.

    z = 1x1 conv D->C on the final patch tokens; Z = bilinear(z -> HxW); class = argmax_c Z.
    Returns logits [C][gh][gw] and classmap [H][W].
    """
    z = ops.conv1x1(_grid(spec, feats[3]), hw["seg_w"], hw["seg_b"])
    Z = ops.bilinear(z, spec.img_h, spec.img_w)
    return {"logits": z, "classmap": _decide(Z)}


def det_head(spec, hw, feats) -> Dict[str, np.ndarray]:
    """Dense detection head: two parallel 3x3 conv towers (D -> Ch, ReLU) on the final
    patch grid; class tower -> 1x1 to the class logits, box tower -> 1x1 to 4 offsets.
    Raw outputs (no sigmoid, decoding or NMS).  Returns logits [K][gh][gw], box [4][gh][gw],
    classmap [gh][gw]."""
    g = _grid(spec, feats[3])
    tc = ops.conv3x3(g, hw["cls_tower_w"], hw["cls_tower_b"], relu=True)
    tb = ops.conv3x3(g, hw["box_tower_w"], hw["box_tower_b"], relu=True)
    logits = ops.conv1x1(tc, hw["cls_w"], hw["cls_b"])
    box = ops.conv1x1(tb, hw["box_w"], hw["box_b"])
    return {"logits": logits, "box": box, "classmap": _decide(logits)}


def depth_head(spec, hw, feats, return_stages: bool = False) -> Dict[str, np.ndarray]:
    """DPT-lite depth head.  Taps deep -> shallow: t_0 = F_3, t_1 = F_2, t_2 = F_1, t_3 = F_0.

    p_s = 1x1 conv D->Ch of t_s on the patch grid; u_s = bilinear(p_s -> 2^s gh x 2^s gw);
    z_s = u_s + y_{s-1} (y_{-1} = 0); y_s = bilinear x2 of ReLU(conv3x3(z_s) + b_s).
    d = 1x1 conv Ch->1 of y_3 (at 16 gh x 16 gw); depth = ReLU(bilinear(d -> H x W)).
    """
    gh, gw = spec.gh, spec.gw
    y = None
    stages = []
    for s in range(4):
        p = ops.conv1x1(_grid(spec, feats[3 - s]), hw[f"proj{s}_w"], hw[f"proj{s}_b"])
        hs, ws = gh << s, gw << s
        u = p if s == 0 else ops.bilinear(p, hs, ws)
        z = u if y is None else u + y
        r = ops.conv3x3(z, hw[f"fuse{s}_w"], hw[f"fuse{s}_b"], relu=True)
        y = ops.bilinear(r, 2 * hs, 2 * ws)
        if return_stages:
            stages.append({"p": p, "z": z, "r": r})
    d = ops.conv1x1(y, hw["out_w"], hw["out_b"])
    pre = ops.bilinear(d, spec.img_h, spec.img_w)[0]
    # "pre_relu" (the map before its final ReLU) is returned beside the result so that a test can tell how much
    # of the signal the ReLU removed
    out = {"depth": np.maximum(pre, 0.0), "pre_relu": pre}
    if return_stages:
        out["stages"] = stages
        out["d16"] = d
    return out


def _rcu(x: np.ndarray, hw, name: str) -> np.ndarray:
    """Residual convolution unit: x + conv3x3(ReLU(conv3x3(ReLU(x)))), both convolutions with bias."""
    t = ops.conv3x3(np.maximum(x, 0.0), hw[name + "_c1_w"], hw[name + "_c1_b"], relu=True)
    return x + ops.conv3x3(t, hw[name + "_c2_w"], hw[name + "_c2_b"])


def dpt_head(spec, hw, feats, return_stages: bool = False) -> Dict[str, np.ndarray]:
    """Dense-prediction-transformer depth head (the structure of the DepthAnythingV2 head that the paper's
    example implementation runs, Sec. "Example implementation"), on one image's four feature maps.

    Width F = head_ch; reassembled widths oc_i = (3 F / 4) 2^i.  Taps shallow -> deep, i = 0..3:
      reassemble   p_i = 1x1 conv D -> oc_i of the patch grid of F_i; then
                   r_0 = transposed conv (kernel = stride = 4) of p_0        -> 4 gh x 4 gw
                   r_1 = transposed conv (kernel = stride = 2) of p_1        -> 2 gh x 2 gw
                   r_2 = p_2                                                 ->   gh x   gw
                   r_3 = 3x3 conv, stride 2, padding 1 of p_3                -> ceil(gh/2) x ceil(gw/2)
      l_i = 3x3 conv oc_i -> F of r_i, no bias.
    Fusion, deep -> shallow, k = 3..0, with s_3 = l_3 and s_k = path_{k+1} + RCU_a(l_k) for k < 3:
      path_k = 1x1 conv F -> F of bilinear_aligned(RCU_b(s_k) -> size of l_{k-1}; for k = 0: twice its size).
    Output: o = 3x3 conv F -> F/2 of path_0; u = bilinear_aligned(o -> H x W);
      depth = ReLU(1x1 conv 32 -> 1 of ReLU(3x3 conv F/2 -> 32 of u)).
    """
    gh, gw = spec.gh, spec.gw
    ls = []
    for i in range(4):
        p = ops.conv1x1(_grid(spec, feats[i]), hw[f"proj{i}_w"], hw[f"proj{i}_b"])
        if i == 0:
            r = ops.conv_transpose(p, hw["up0_w"], hw["up0_b"], 4)
        elif i == 1:
            r = ops.conv_transpose(p, hw["up1_w"], hw["up1_b"], 2)
        elif i == 2:
            r = p
        else:
            r = ops.conv3x3_s2(p, hw["down3_w"], hw["down3_b"])
        ls.append(ops.conv3x3(r, hw[f"rn{i}_w"], None))
    path = None
    paths = []
    for k in (3, 2, 1, 0):
        s = ls[k] if path is None else path + _rcu(ls[k], hw, f"fuse{k}_a")
        y = _rcu(s, hw, f"fuse{k}_b")
        size = (ls[k - 1].shape[1], ls[k - 1].shape[2]) if k > 0 else (2 * y.shape[1], 2 * y.shape[2])
        path = ops.conv1x1(ops.bilinear_ac(y, *size), hw[f"fuse{k}_out_w"], hw[f"fuse{k}_out_b"])
        paths.append(path)
    o = ops.conv3x3(path, hw["head1_w"], hw["head1_b"])
    u = ops.bilinear_ac(o, spec.img_h, spec.img_w)
    v = ops.conv3x3(u, hw["head2_w"], hw["head2_b"], relu=True)
    pre = ops.conv1x1(v, hw["head3_w"], hw["head3_b"])[0]
    out = {"depth": np.maximum(pre, 0.0), "pre_relu": pre}
    if return_stages:
        out["l"] = ls
        out["paths"] = paths
        out["o"] = o
    return out
