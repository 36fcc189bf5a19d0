"""Seeded synthetic inputs for the Visual Perception Engine hot path.

This module only *draws numbers*: model shapes, random weights, synthetic camera
frames and the flat weight-blob layout.  It holds none of the method's arithmetic
(no layer, no attention, no convolution) and is the only code that both the CPU
oracle's tests and the HIP path's tests/bench use.

The paper (Sec. "Example implementation") runs trained DINOv2 / DepthAnythingV2 /
linear-seg / detection weights on 1920x1080 camera streams; none of that data is
available, so these generators stand in for it:

* weights: every tensor ~ N(0, 0.02^2) truncated to +-2 std by rejection (the full DPT head: kernels
  N(0, 2 / fan_in), biases N(0, 0.1^2), same truncation, see _dpt_std);
  LayerNorm gains are 1 + that, LayerScale vectors are the constant 0.1;
  for the bf16 configurations every value is rounded once to the nearest bf16
  (ties to even) so both sides start from the same stored parameters.
* frames: per channel a sum of 8 random 2-D sinusoids (amplitude U(0.5,1),
  frequency U(-4,4) cycles per image, phase U(0,2pi)) plus N(0, 0.05^2) noise,
  then normalised per channel to zero mean / unit std.
* sequences: the analytic field evaluated at an accumulating integer shift of
  0..4 px per axis per frame, with fresh noise each frame.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np

PATCH = 14
HEAD_DIM = 64

MLP_GELU = 0
MLP_SWIGLU = 1

HEAD_SEG = 0
HEAD_DEPTH = 1
HEAD_DET = 2
HEAD_DPT = 3


@dataclass(frozen=True)
class ModelSpec:
    """Shapes of one encoder + heads configuration."""
    name: str
    dim: int
    depth: int
    heads: int
    mlp_hidden: int
    mlp_kind: int = MLP_GELU
    registers: int = 0
    batch: int = 1
    img_h: int = 224
    img_w: int = 224
    dtype: str = "bf16"          # "f32" or "bf16": arithmetic type of the GPU path
    taps: Tuple[int, int, int, int] = (3, 6, 9, 12)   # 1-based block indices
    seg_classes: int = 21
    det_classes: int = 80
    head_ch: int = 256
    ln_eps: float = 1e-6
    head_dim: int = HEAD_DIM

    @property
    def gh(self) -> int:
        return self.img_h // PATCH

    @property
    def gw(self) -> int:
        return self.img_w // PATCH

    @property
    def patches(self) -> int:
        return self.gh * self.gw

    @property
    def tokens(self) -> int:
        return 1 + self.registers + self.patches

    @property
    def fc1_out(self) -> int:
        return self.mlp_hidden * (2 if self.mlp_kind == MLP_SWIGLU else 1)


# The five benchmark configurations (index 0 = the small fp32 case).
CONFIGS: Dict[str, ModelSpec] = {
    "cfg1": ModelSpec("vits14_f32_224", 384, 12, 6, 1536, batch=1, img_h=224, img_w=224, dtype="f32"),
    "cfg2": ModelSpec("vits14_bf16_476x630", 384, 12, 6, 1536, batch=1, img_h=476, img_w=630),
    "cfg3": ModelSpec("vitb14_bf16_518", 768, 12, 12, 3072, batch=1, img_h=518, img_w=518),
    "cfg4": ModelSpec("vitl14_bf16_518_b4", 1024, 24, 16, 4096, registers=4, batch=4, img_h=518, img_w=518,
                      taps=(6, 12, 18, 24)),
    "cfg5": ModelSpec("vitg14_bf16_518_b8", 1536, 40, 24, 4096, mlp_kind=MLP_SWIGLU, registers=4, batch=8,
                      img_h=518, img_w=518, taps=(10, 20, 30, 40), seg_classes=150),
}

# Seeds per configuration: (weights, first image).
SEEDS = {"cfg1": (1001, 2001), "cfg2": (1002, 2002), "cfg3": (1003, 2003), "cfg4": (1004, 2004),
         "cfg5": (1005, 2008)}
SHIFT_SEED_CFG3 = 3003


def small_spec(name: str = "tiny", **kw) -> ModelSpec:
    """A reduced model with the structure of the benchmark ones, for fast tests."""
    base = dict(dim=128, depth=4, heads=2, mlp_hidden=256, batch=1, img_h=56, img_w=84, taps=(1, 2, 3, 4),
                seg_classes=21, det_classes=80, head_ch=64, dtype="bf16")
    base.update(kw)
    return ModelSpec(name, **base)


def with_(spec: ModelSpec, **kw) -> ModelSpec:
    return replace(spec, **kw)


# --------------------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bfloat16 (ties to even); result stays fp32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    r &= np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(np.shape(a))


# --------------------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------------------
def _trunc_normal_into(rng: np.random.Generator, out: np.ndarray, std: float = 0.02) -> None:
    """Fill the flat fp32 array `out` with N(0, std^2) truncated to +-2 std (by rejection)."""
    rng.standard_normal(out.size, dtype=np.float32, out=out)
    bad = np.flatnonzero(np.abs(out) > 2.0)
    while bad.size:
        out[bad] = rng.standard_normal(bad.size, dtype=np.float32)
        bad = bad[np.abs(out[bad]) > 2.0]
    out *= np.float32(std)


def backbone_layout(spec: ModelSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of the backbone tensors, in weight-blob order.

    Linear weights are stored [in][out] (y = x W + b); the patch-embed kernel is
    [D][3][14][14].  qkv columns: all q heads, then k, then v; head i owns columns
    64*i..64*i+63 of each third.  SwiGLU fc1 columns: the gate half (a) then the
    linear half (b).
    """
    D, P, R = spec.dim, spec.patches, spec.registers
    out: List[Tuple[str, Tuple[int, ...]]] = [
        ("patch_w", (D, 3, PATCH, PATCH)), ("patch_b", (D,)),
        ("cls", (D,)), ("reg", (R, D)), ("pos", (1 + P, D)),
    ]
    for l in range(spec.depth):
        p = f"blk{l}."
        out += [
            (p + "ln1_g", (D,)), (p + "ln1_b", (D,)),
            (p + "qkv_w", (D, 3 * D)), (p + "qkv_b", (3 * D,)),
            (p + "proj_w", (D, D)), (p + "proj_b", (D,)),
            (p + "ls1", (D,)),
            (p + "ln2_g", (D,)), (p + "ln2_b", (D,)),
            (p + "fc1_w", (D, spec.fc1_out)), (p + "fc1_b", (spec.fc1_out,)),
            (p + "fc2_w", (spec.mlp_hidden, D)), (p + "fc2_b", (D,)),
            (p + "ls2", (D,)),
        ]
    out += [("norm_g", (D,)), ("norm_b", (D,))]
    return out


def head_layout(spec: ModelSpec, kind: int) -> List[Tuple[str, Tuple[int, ...]]]:
    """Names and shapes of one head's tensors, in weight-blob order.

    Convolution kernels are [Cout][Cin][kh][kw]; 1x1 convolutions are [Cout][Cin].
    """
    D, Ch = spec.dim, spec.head_ch
    if kind == HEAD_SEG:
        return [("seg_w", (spec.seg_classes, D)), ("seg_b", (spec.seg_classes,))]
    if kind == HEAD_DET:
        return [
            ("cls_tower_w", (Ch, D, 3, 3)), ("cls_tower_b", (Ch,)),
            ("box_tower_w", (Ch, D, 3, 3)), ("box_tower_b", (Ch,)),
            ("cls_w", (spec.det_classes, Ch)), ("cls_b", (spec.det_classes,)),
            ("box_w", (4, Ch)), ("box_b", (4,)),
        ]
    if kind == HEAD_DEPTH:
        out = []
        for s in range(4):   # s = 0 is the deepest tap (final tokens)
            out += [(f"proj{s}_w", (Ch, D)), (f"proj{s}_b", (Ch,))]
        for s in range(4):
            out += [(f"fuse{s}_w", (Ch, Ch, 3, 3)), (f"fuse{s}_b", (Ch,))]
        out += [("out_w", (1, Ch)), ("out_b", (1,))]
        return out
    if kind == HEAD_DPT:
        F = Ch
        oc = [3 * F // 4 << i for i in range(4)]
        out = []
        for i in range(4):   # i = 0 is the shallowest tap
            out += [(f"proj{i}_w", (oc[i], D)), (f"proj{i}_b", (oc[i],))]
        out += [("up0_w", (oc[0], oc[0], 4, 4)), ("up0_b", (oc[0],)),       # transposed convolutions: [Cin][Cout][k][k]
                ("up1_w", (oc[1], oc[1], 2, 2)), ("up1_b", (oc[1],)),
                ("down3_w", (oc[3], oc[3], 3, 3)), ("down3_b", (oc[3],))]
        for i in range(4):
            out += [(f"rn{i}_w", (F, oc[i], 3, 3))]
        for k in (3, 2, 1, 0):
            for unit in (("b",) if k == 3 else ("a", "b")):
                for c in ("c1", "c2"):
                    out += [(f"fuse{k}_{unit}_{c}_w", (F, F, 3, 3)), (f"fuse{k}_{unit}_{c}_b", (F,))]
            out += [(f"fuse{k}_out_w", (F, F)), (f"fuse{k}_out_b", (F,))]
        out += [("head1_w", (F // 2, F, 3, 3)), ("head1_b", (F // 2,)),
                ("head2_w", (32, F // 2, 3, 3)), ("head2_b", (32,)),
                ("head3_w", (1, 32)), ("head3_b", (1,))]
        return out
    raise ValueError(f"unknown head kind {kind}")


def _dpt_std(name: str, shape) -> float:
    """Standard deviation of a DPT-head tensor: convolution kernels sqrt(2 / fan_in) (fan_in = inputs that feed
    one output value: Cin k k, or Cin alone for the stride = kernel transposed convolutions, stored [Cin][Cout][k][k]),
    so that the activations keep their size through the ~20 layers of the head and every layer's contribution is
    visible in the output; biases 0.1."""
    if name.endswith("_b"):
        return 0.1
    fan_in = shape[0] if name.startswith("up") else int(np.prod(shape[1:]))
    return float(np.sqrt(2.0 / fan_in))


def _fill(layout, seed: int, quantize: bool, std_of=None) -> Dict[str, np.ndarray]:
    """All tensors of a layout, generated straight into one flat blob (key "__blob__"); the named
    entries are views of it.  Tensor i draws from its own stream PCG64(SeedSequence([seed, i])), so
    tensors can be filled in parallel and do not depend on each other's sizes."""
    sizes = [int(np.prod(shape)) for _, shape in layout]
    blob = np.empty(int(sum(sizes)), dtype=np.float32)
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)

    def one(i: int) -> None:
        name, _ = layout[i]
        dst = blob[offs[i]:offs[i + 1]]
        leaf = name.split(".")[-1]
        if leaf in ("ls1", "ls2"):
            dst[:] = np.float32(0.1)
        else:
            _trunc_normal_into(np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, i]))), dst,
                               0.02 if std_of is None else std_of(name, layout[i][1]))
            if leaf in ("ln1_g", "ln2_g", "norm_g"):
                dst += np.float32(1.0)
        if quantize:
            dst[:] = round_bf16(dst)

    workers = max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(one, range(len(layout))))
    w: Dict[str, np.ndarray] = {name: blob[offs[i]:offs[i + 1]].reshape(shape) for i, (name, shape) in enumerate(layout)}
    w["__blob__"] = blob
    return w


def make_backbone_weights(spec: ModelSpec, seed: int) -> Dict[str, np.ndarray]:
    return _fill(backbone_layout(spec), seed, spec.dtype == "bf16")


def make_head_weights(spec: ModelSpec, kind: int, seed: int) -> Dict[str, np.ndarray]:
    return _fill(head_layout(spec, kind), seed * 7919 + 17 * (kind + 1), spec.dtype == "bf16",
                 _dpt_std if kind == HEAD_DPT else None)


def pack(layout, w: Dict[str, np.ndarray]) -> np.ndarray:
    """The flat fp32 blob the C ABI takes: the tensors of `layout` concatenated in order.  A dict made by
    make_*_weights already is one blob (unless an entry was replaced), which is returned without a copy."""
    blob = w.get("__blob__")
    if blob is not None:
        off, same = 0, True
        for name, shape in layout:
            a = w[name]
            n = int(np.prod(shape))
            same = same and a.dtype == np.float32 and tuple(a.shape) == tuple(shape) and a.size == n and \
                (n == 0 or (a.base is not None and a.__array_interface__["data"][0] == blob.__array_interface__["data"][0] + 4 * off))
            off += n
        if same and off == blob.size:
            return blob
    parts = []
    for name, shape in layout:
        a = np.asarray(w[name], dtype=np.float32)
        assert tuple(a.shape) == tuple(shape), (name, a.shape, shape)
        parts.append(a.reshape(-1))
    return np.ascontiguousarray(np.concatenate(parts)) if parts else np.zeros(0, np.float32)


def pack_backbone(spec: ModelSpec, w) -> np.ndarray:
    return pack(backbone_layout(spec), w)


def pack_head(spec: ModelSpec, kind: int, w) -> np.ndarray:
    return pack(head_layout(spec, kind), w)


def blob_floats(layout) -> int:
    return int(sum(int(np.prod(s)) for _, s in layout))


# --------------------------------------------------------------------------------------
# frames
# --------------------------------------------------------------------------------------
@dataclass
class Field:
    """Analytic part of one synthetic camera view: 3 channels x 8 sinusoids."""
    amp: np.ndarray
    fx: np.ndarray
    fy: np.ndarray
    phase: np.ndarray
    h: int
    w: int

    def evaluate(self, dx: int = 0, dy: int = 0) -> np.ndarray:
        y = (np.arange(self.h, dtype=np.float64) + dy)[:, None] / self.h
        x = (np.arange(self.w, dtype=np.float64) + dx)[None, :] / self.w
        out = np.zeros((3, self.h, self.w), dtype=np.float64)
        for c in range(3):
            for k in range(self.amp.shape[1]):
                out[c] += self.amp[c, k] * np.sin(
                    2.0 * np.pi * (self.fx[c, k] * x + self.fy[c, k] * y) + self.phase[c, k])
        return out


def make_field(h: int, w: int, rng: np.random.Generator, terms: int = 8) -> Field:
    return Field(amp=rng.uniform(0.5, 1.0, (3, terms)), fx=rng.uniform(-4.0, 4.0, (3, terms)),
                 fy=rng.uniform(-4.0, 4.0, (3, terms)), phase=rng.uniform(0.0, 2.0 * np.pi, (3, terms)),
                 h=h, w=w)


def _finish(clean: np.ndarray, rng: np.random.Generator) -> np.ndarray:
    img = clean + rng.normal(0.0, 0.05, clean.shape)
    img = (img - img.mean(axis=(1, 2), keepdims=True)) / img.std(axis=(1, 2), keepdims=True)
    return img.astype(np.float32)


def make_image(h: int, w: int, seed: int) -> np.ndarray:
    """One normalised frame [3, h, w] fp32."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return _finish(make_field(h, w, rng).evaluate(), rng)


# the usual ImageNet statistics, as used in front of DINOv2-style backbones (data, not arithmetic)
CAMERA_MEAN = (0.485, 0.456, 0.406)
CAMERA_STD = (0.229, 0.224, 0.225)


def make_camera_frame(h: int, w: int, seed: int) -> np.ndarray:
    """One raw camera frame [h, w, 3] uint8 (interleaved RGB): the same smooth field + sensor noise as
    make_image, mapped to 0..255 with some clipping at both ends, as real frames have."""
    rng = np.random.Generator(np.random.PCG64(seed))
    clean = make_field(h, w, rng).evaluate()
    img = clean + rng.normal(0.0, 0.05, clean.shape)
    img = 128.0 + 48.0 * img                       # field amplitude is a few units: reaches past 0 and 255
    return np.ascontiguousarray(np.clip(np.rint(img), 0, 255).astype(np.uint8).transpose(1, 2, 0))


def make_batch(spec: ModelSpec, seed: int) -> np.ndarray:
    """[B, 3, H, W] fp32; batch element b (a camera view) uses seed + b."""
    return np.stack([make_image(spec.img_h, spec.img_w, seed + b) for b in range(spec.batch)])


def make_sequence(spec: ModelSpec, seed: int, shift_seed: int, frames: int, only=None):
    """Generator of [B, 3, H, W] frames: each one is the previous view translated by a
    random 0..4 px per axis (accumulated, evaluated analytically) plus new noise.

    only: optional set of frame indices to materialise; other frames yield None but still
    advance the shift and noise generators, so frame t is the same whatever `only` is."""
    rngs = [np.random.Generator(np.random.PCG64(seed + b)) for b in range(spec.batch)]
    fields = [make_field(spec.img_h, spec.img_w, r) for r in rngs]
    srng = np.random.Generator(np.random.PCG64(shift_seed))
    dx = dy = 0
    shape = (3, spec.img_h, spec.img_w)
    for t in range(frames):
        if t:
            dx += int(srng.integers(0, 5))
            dy += int(srng.integers(0, 5))
        if only is None or t in only:
            yield np.stack([_finish(f.evaluate(dx, dy), r) for f, r in zip(fields, rngs)])
        else:
            for r in rngs:
                r.normal(0.0, 0.05, shape)      # keep the noise stream in step
            yield None
