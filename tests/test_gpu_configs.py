"""GPU checks at the shapes of benchmark configurations 3, 4 and 5.

cfg 3 (ViT-B/14, 518x518, rates 1/2/3 over a 300-frame sequence) is run whole: every frame is pushed
through the engine without host synchronisation, run counts are exact, and frames 0, 6 and 299 are
compared with the oracle.  cfgs 4 and 5 (ViT-L batch 4 with 24 blocks, ViT-g batch 8 with 40 blocks) are run
whole as well, as the benchmark launches them (HIP graphs), and compared with the oracle at full depth on
the first and the last batch element (the fp64 loops take about 15 s and 50 s for one image; the last rows of
the batch can go through another tile shape than the leading ones); the other batch elements are tied
to these by batch independence: swapping two views swaps the results (bit for bit with one tile shape per
GEMM, to rounding otherwise).  The four-block cuts
of the same shapes stay as the quick variant (they also check the last batch element against the oracle).
"""
import numpy as np
import pytest
import torch

import paper_2508_11584_amd as vpe
import vpe_inputs as vi
from helpers import depth_errs, depth_gate, make_engine, relerr
from oracle import model
from test_gpu_parity import check_all

pytestmark = pytest.mark.gpu


def test_cfg3_vitb_sequence_rates_and_parity():
    spec = vi.CONFIGS["cfg3"]
    wseed, iseed = vi.SEEDS["cfg3"]
    eng, w, hw = make_engine(spec, wseed, kinds=("depth", "seg", "det"), every_n=(1, 2, 3), flags=vpe.VPE_FLAG_GRAPHS)
    check = {0, 6, 299}                       # frame 6 is due for all three heads, 299 only for depth
    n = 300
    pool = []                                 # a few distinct resident frames for the unchecked steps
    got = {}
    for t, fr in enumerate(vi.make_sequence(spec, iseed, vi.SHIFT_SEED_CFG3, n, only=check | set(range(1, 5)))):
        if fr is not None:
            pool.append((t, torch.from_numpy(fr).cuda(), fr))
        tt, dev, host = pool[-1] if fr is not None else pool[1 + t % 4]
        fh = eng.encode(dev)
        rcs = [eng.run_head(h, fh) for h in range(3)]
        assert rcs == [0, 0 if t % 2 == 0 else 1, 0 if t % 3 == 0 else 1]
        if t in check:
            eng.sync()
            got[t] = {"host": host, "feat3": eng.feat_view(fh, 3).float().cpu().numpy()[0],
                      "depth": eng.head_output(0, 0).cpu().numpy()[0].copy(),
                      "seg": eng.head_output(1, 1).cpu().numpy()[0].copy() if t % 2 == 0 else None,
                      "det": eng.head_output(2, 0).cpu().numpy()[0].copy() if t % 3 == 0 else None}
    eng.sync()
    frames, runs, skips = eng.stats()
    assert frames == 300 and runs == [300, 150, 100] and skips == [0, 150, 200]
    eng.close()
    for t, g in got.items():
        feats = model.encode_image(spec, w, g["host"][0])
        de = depth_errs(g["depth"], model.depth_head(spec, hw[0], feats))
        e = {"feat3": relerr(g["feat3"], feats[3]), "depth": de["stated"], "depth_pre_relu": de["pre_relu"],
             "depth_positive": de["positive"]}
        if g["seg"] is not None:
            e["seg_agree"] = float(np.mean(g["seg"] == model.seg_head(spec, hw[1], feats)["classmap"]))
        if g["det"] is not None:
            o = model.det_head(spec, hw[2], feats)
            e["det_logits"] = relerr(g["det"][..., :80].transpose(2, 0, 1), o["logits"])
        print("cfg3 frame", t, {k: round(v, 5) for k, v in e.items()}, flush=True)
        assert e["feat3"] <= 2e-2 and depth_gate(de, 2e-2), (e, de)
        assert e.get("seg_agree", 1.0) >= 0.99 and e.get("det_logits", 0.0) <= 2e-2


def test_cfg4_shapes_vitl_batch4_registers_four_blocks():
    spec = vi.with_(vi.CONFIGS["cfg4"], name="vitl_shapes_4blk", depth=4, taps=(1, 2, 3, 4))
    check_all(spec, 1004, 2004, batch_check=(0, 3))


def test_cfg5_shapes_vitg_swiglu_batch8_four_blocks():
    spec = vi.with_(vi.CONFIGS["cfg5"], name="vitg_shapes_4blk", depth=4, taps=(1, 2, 3, 4))
    check_all(spec, 1005, 2008, batch_check=(0, 7))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg", ["cfg4", "cfg5"])
def test_full_depth_large_configs_match_the_oracle_and_are_consistent(cfg):
    spec = vi.CONFIGS[cfg]
    wseed, iseed = vi.SEEDS[cfg]

    def on_device(eng, imgs, fh0, feats0, outs0):
        # determinism (the second pass lands in the other ring slot and replays its own graphs)
        fh = eng.encode(torch.from_numpy(imgs).cuda())
        for h in range(3):
            assert eng.run_head(h, fh) == 0
        eng.sync()
        feat = eng.feat_view(fh, 3).clone()
        depth = eng.head_output(1, 0).clone()
        assert np.array_equal(feat.float().cpu().numpy(), feats0[3])
        assert np.array_equal(depth.cpu().numpy(), outs0[1][0])
        assert np.array_equal(eng.head_output(0, 1).cpu().numpy(), outs0[0][1])
        assert torch.isfinite(feat.float()).all() and torch.isfinite(depth).all() and depth.min() >= 0
        assert not torch.equal(feat[0], feat[1])                  # different views give different features
        assert int(outs0[0][1].max()) < spec.seg_classes
        # batch independence at full depth: a batch with two views swapped gives the swapped results.  Views that
        # keep their place are bit-identical; the last rows of a batch may go through another tile shape than the
        # leading ones (a GEMM whose tile count is just above whole rounds of the CUs is launched in two parts), so
        # a view that moves to or from the last place agrees to rounding (bit-identity of moved views with
        # one tile shape per GEMM: test_views_do_not_depend_on_their_place_in_the_batch)
        perm = list(range(spec.batch))
        perm[0], perm[-1] = perm[-1], perm[0]
        fh = eng.encode(torch.from_numpy(np.ascontiguousarray(imgs[perm])).cuda())
        for h in range(3):
            eng.run_head(h, fh)
        eng.sync()
        f2, d2 = eng.feat_view(fh, 3), eng.head_output(1, 0)
        for b in range(1, spec.batch - 1):
            assert torch.equal(f2[b], feat[b]) and torch.equal(d2[b], depth[b])
        for a, b in ((0, spec.batch - 1), (spec.batch - 1, 0)):
            ef = relerr(f2[a].float().cpu().numpy(), feat[b].float().cpu().numpy())
            ed = relerr(d2[a].cpu().numpy(), depth[b].cpu().numpy())
            print(f"{cfg}: view {b} moved to place {a}: feature difference {ef:.2e}, depth difference {ed:.2e}")
            assert ef <= 2e-2 and ed <= 2e-2

    check_all(spec, wseed, iseed, flags=vpe.VPE_FLAG_GRAPHS, batch_check=(0, spec.batch - 1), on_device=on_device)


@pytest.mark.parametrize("cfg", ["cfg4", "cfg5"])
def test_views_do_not_depend_on_their_place_in_the_batch(cfg, monkeypatch):
    """With one tile shape per GEMM (the two-part launch switched off when the engine is created) every view's
    features and depth map are bit-identical wherever the view sits in the batch, at full depth."""
    monkeypatch.setenv("VPE_NO_ROW_SPLIT", "1")
    spec = vi.CONFIGS[cfg]
    wseed, iseed = vi.SEEDS[cfg]
    eng, _, _ = make_engine(spec, wseed, flags=vpe.VPE_FLAG_GRAPHS)
    imgs = vi.make_batch(spec, iseed)
    perm = list(range(spec.batch))
    perm[0], perm[-1] = perm[-1], perm[0]
    got = []
    for order in (list(range(spec.batch)), perm):
        fh = eng.encode(torch.from_numpy(np.ascontiguousarray(imgs[order])).cuda())
        for h in range(3):
            assert eng.run_head(h, fh) == 0
        eng.sync()
        got.append((eng.feat_view(fh, 3).clone(), eng.head_output(1, 0).clone()))
    eng.close()
    for place, view in enumerate(perm):
        assert torch.equal(got[1][0][place], got[0][0][view]) and torch.equal(got[1][1][place], got[0][1][view])
    assert not torch.equal(got[0][0][0], got[0][0][-1])
