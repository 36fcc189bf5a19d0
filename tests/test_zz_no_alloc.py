"""vpe_run_head_static (the head run for callers that cannot allocate: intermediate buffers in the library's static
device array, no graph instantiation) against vpe_run_head, through the C ABI: same kernels on the same features,
so every output must be bit-identical; two calls in a row, the second on a smaller model input."""
import pytest
import torch

import paper_2508_11584_amd as vpe
import vpe_inputs as vi
from helpers import make_engine

pytestmark = pytest.mark.gpu

KINDS = ("seg", "depth", "det")
BIG = vi.ModelSpec("static_big", dim=128, depth=4, heads=2, mlp_hidden=256, img_h=98, img_w=154, taps=(1, 2, 3, 4),
                   head_ch=64, dtype="bf16", batch=2)
SMALL = vi.with_(BIG, name="static_small", img_h=42, img_w=70, batch=1)


def outputs(eng):
    return [eng.head_output(h, w).clone() for h, w in ((0, 0), (0, 1), (1, 0), (2, 0), (2, 1))]


def free_bytes():
    return torch.cuda.mem_get_info()[0]


def run_both(spec, seed, flags):
    eng, _, _ = make_engine(spec, seed, kinds=KINDS, flags=flags)
    img = torch.from_numpy(vi.make_batch(spec, seed + 50)).cuda()
    fh = eng.encode(img)
    for h in range(3):
        assert eng.run_head(h, fh) == vpe.VPE_OK
    eng.sync()
    ref = outputs(eng)
    for h in range(3):                      # poison the outputs so that a run that writes nothing cannot pass
        for w in range(2 if h != 1 else 1):
            eng.head_output(h, w).fill_(7)
    torch.cuda.synchronize()
    before = (free_bytes(), torch.cuda.memory_allocated())
    for h in range(3):                      # one after the other on the heads' streams: the array is shared
        assert vpe.vpe_run_head_static(eng.handle, h, fh) == vpe.VPE_OK
        eng.wait_head(h)
    eng.sync()
    assert (free_bytes(), torch.cuda.memory_allocated()) == before          # nothing was allocated on the device
    got = outputs(eng)
    for a, b in zip(ref, got):
        assert torch.equal(a, b)
    assert eng.stats()[1] == [2, 2, 2]      # counted as runs like any other
    return eng


def test_static_scratch_head_runs_match_the_workspace_ones_twice_in_a_row_second_smaller():
    big = run_both(BIG, 61, vpe.VPE_FLAG_GRAPHS)       # also: never a graph replay, even on an engine with graphs
    small = run_both(SMALL, 62, 0)                     # the array now holds the larger run's leftovers
    # and the larger one again after the smaller, on the same engine and a new frame
    img = torch.from_numpy(vi.make_batch(BIG, 999)).cuda()
    fh = big.encode(img)
    for h in range(3):
        assert vpe.vpe_run_head_static(big.handle, h, fh, None) == vpe.VPE_OK
        big.wait_head(h)
    got = outputs(big)
    for h in range(3):
        assert big.run_head(h, fh) == vpe.VPE_OK
    big.sync()
    for a, b in zip(got, outputs(big)):
        assert torch.equal(a, b)
    small.close()
    big.close()


def test_static_scratch_rejects_what_does_not_fit_and_keeps_the_rate_rules():
    spec = vi.CONFIGS["cfg2"]                          # its depth head needs about 100 MB of intermediates
    eng, _, _ = make_engine(spec, 1002, kinds=KINDS, every_n=(1, 1, 2))
    img = torch.from_numpy(vi.make_batch(spec, 2002)).cuda()
    fh0 = eng.encode(img)
    with pytest.raises(vpe.VpeError, match="static array holds 8388608"):
        vpe.vpe_run_head_static(eng.handle, 1, fh0)
    assert vpe.vpe_run_head_static(eng.handle, 2, fh0) == vpe.VPE_OK        # the detection head fits (1.6 MB)
    eng.wait_head(2)
    det = eng.head_output(2, 0).clone()
    assert eng.run_head(2, fh0) == vpe.VPE_OK
    eng.sync()
    assert torch.equal(det, eng.head_output(2, 0))
    fh1 = eng.encode(img)
    assert vpe.vpe_run_head_static(eng.handle, 2, fh1) == vpe.VPE_SKIPPED   # every 2nd frame only
    eng.encode(img)
    with pytest.raises(vpe.VpeError) as ei:                                 # ring of two: frame 0's slot is gone
        vpe.vpe_run_head_static(eng.handle, 0, fh0)
    assert ei.value.code == vpe.VPE_ESTALE
    eng.close()
