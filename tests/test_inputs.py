"""The seeded input generators: value ranges, determinism, blob layout."""
import numpy as np
import torch

import vpe_inputs as vi


def test_round_bf16_matches_library_rounding():
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.normal(size=4096).astype(np.float32) * 0.02,
                        np.array([1.0, 1.00390625, 1.01171875, -0.0, 3.3895314e38], np.float32)])
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(vi.round_bf16(a), ref)


def test_weights_are_truncated_seeded_and_bf16_exact():
    spec = vi.small_spec()
    w = vi.make_backbone_weights(spec, 7)
    w2 = vi.make_backbone_weights(spec, 7)
    for k, v in w.items():
        assert np.array_equal(v, w2[k]), k
        if k == "__blob__":
            continue
        leaf = k.split(".")[-1]
        if leaf in ("ls1", "ls2"):
            assert np.all(v == vi.round_bf16(np.float32(0.1)))
        elif leaf.endswith("_g"):
            assert np.all(np.abs(v - 1.0) <= 0.0401)
        else:
            assert np.all(np.abs(v) <= 0.0401), k
        assert np.array_equal(v, vi.round_bf16(v))
    big = w["blk0.fc1_w"]
    assert 0.015 < big.std() < 0.02          # std of N(0,0.02^2) truncated at 2 sigma = 0.0176
    f32 = vi.make_backbone_weights(vi.with_(spec, dtype="f32"), 7)
    assert not np.array_equal(f32["pos"], vi.round_bf16(f32["pos"]))


def test_blob_layout_is_the_concatenation_in_order():
    spec = vi.small_spec(registers=2, mlp_kind=vi.MLP_SWIGLU)
    w = vi.make_backbone_weights(spec, 9)
    blob = vi.pack_backbone(spec, w)
    assert blob.dtype == np.float32 and blob.size == vi.blob_floats(vi.backbone_layout(spec))
    off = 0
    for name, shape in vi.backbone_layout(spec):
        n = int(np.prod(shape))
        assert np.array_equal(blob[off:off + n], w[name].reshape(-1)), name
        off += n
    assert w["blk0.fc1_w"].shape == (spec.dim, 2 * spec.mlp_hidden)
    assert vi.pack_backbone(spec, w) is w["__blob__"]                       # no copy when nothing was replaced
    w3 = dict(w)
    w3["pos"] = w["pos"] * 2                                                # a replaced tensor forces a re-pack
    b3 = vi.pack_backbone(spec, w3)
    assert b3 is not w["__blob__"] and b3.size == blob.size and not np.array_equal(b3, blob)
    for kind in (vi.HEAD_SEG, vi.HEAD_DEPTH, vi.HEAD_DET):
        hw = vi.make_head_weights(spec, kind, 9)
        assert vi.pack_head(spec, kind, hw).size == vi.blob_floats(vi.head_layout(spec, kind))


def test_images_are_normalised_per_channel_and_seeded():
    a = vi.make_image(56, 84, 5)
    assert a.shape == (3, 56, 84) and a.dtype == np.float32
    assert np.allclose(a.mean(axis=(1, 2)), 0, atol=1e-5) and np.allclose(a.std(axis=(1, 2)), 1, atol=1e-5)
    assert np.array_equal(a, vi.make_image(56, 84, 5))
    assert not np.array_equal(a, vi.make_image(56, 84, 6))
    spec = vi.small_spec(batch=3)
    b = vi.make_batch(spec, 5)
    assert b.shape == (3, 3, 56, 84) and np.array_equal(b[0], a) and not np.array_equal(b[1], a)


def test_sequence_frames_are_shifted_views():
    spec = vi.small_spec()
    frames = list(vi.make_sequence(spec, 5, 6, 4))
    assert len(frames) == 4 and frames[0].shape == (1, 3, 56, 84)
    # consecutive frames stay strongly correlated (small translation), but are not equal (new noise)
    for a, b in zip(frames, frames[1:]):
        c = np.corrcoef(a.ravel(), b.ravel())[0, 1]
        assert 0.5 < c < 0.9999


def test_benchmark_config_shapes():
    c = vi.CONFIGS
    assert (c["cfg1"].tokens, c["cfg2"].tokens, c["cfg3"].tokens, c["cfg4"].tokens, c["cfg5"].tokens) == \
        (257, 1531, 1370, 1374, 1374)
    assert c["cfg2"].gh == 34 and c["cfg2"].gw == 45
    assert all(s.dim == s.heads * 64 for s in c.values())
    assert c["cfg5"].fc1_out == 8192 and c["cfg5"].seg_classes == 150


def test_sequence_frame_selection_does_not_change_the_frames():
    spec = vi.small_spec()
    full = list(vi.make_sequence(spec, 5, 6, 6))
    part = list(vi.make_sequence(spec, 5, 6, 6, only={0, 4, 5}))
    assert part[1] is None and part[2] is None and part[3] is None
    for t in (0, 4, 5):
        assert np.array_equal(full[t], part[t])
