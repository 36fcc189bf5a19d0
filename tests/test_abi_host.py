"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, validates
configurations, and its host-side scheduling logic (slot ring, rates, staleness, counters)
behaves as the header says.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2508_11584_amd as vpe
import vpe_inputs as vi
from helpers import make_engine

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "vpe.h")).read()
    names = set(re.findall(r"\b(vpe_[a-z_]+)\s*\(", hdr))
    assert {"vpe_create", "vpe_encode", "vpe_run_head", "vpe_set_head_rate"} <= names
    L = vpe.lib()
    for n in sorted(names):
        assert hasattr(L, n), n


def test_binding_structs_match_the_header_layout(tmp_path):
    # the header compiled as plain C (it must be one) reports size and field offsets of every struct;
    # the ctypes mirrors must agree field by field
    structs = {"vpe_feat": vpe.binding.vpe_feat, "vpe_backbone_cfg": vpe.binding.vpe_backbone_cfg,
               "vpe_head_cfg": vpe.binding.vpe_head_cfg}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "vpe.h"', 'int main(void) {']
    for name, st in structs.items():
        lines.append(f'printf("{name} size %zu\\n", sizeof({name}));')
        for f, _ in st._fields_:
            lines.append(f'printf("{name} {f} %zu\\n", offsetof({name}, {f}));')
    lines += ["return 0; }"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = 0
    for ln in filter(None, out):
        name, field, val = ln.split()
        st = structs[name]
        assert int(val) == (C.sizeof(st) if field == "size" else getattr(st, field).offset), ln
        seen += 1
    assert seen == sum(len(st._fields_) + 1 for st in structs.values())


def test_product_does_not_import_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2508_11584_amd")):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt, os.path.join(dirpath, f)
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            assert "paper_2508_11584_amd" not in open(os.path.join(ROOT, "oracle", f)).read()


def _cfg(spec, blob, **over):
    c = vpe.binding.vpe_backbone_cfg()
    c.dim, c.depth, c.heads, c.mlp_hidden, c.mlp_kind = spec.dim, spec.depth, spec.heads, spec.mlp_hidden, spec.mlp_kind
    c.registers, c.img_h, c.img_w, c.batch, c.dtype = spec.registers, spec.img_h, spec.img_w, spec.batch, 1
    c.taps = (C.c_int32 * 4)(*spec.taps)
    c.ring_slots, c.flags, c.ln_eps = 2, vpe.VPE_FLAG_HOST_ONLY, 1e-6
    c.weights, c.weights_bytes = blob.ctypes.data, blob.nbytes
    for k, v in over.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("over,needle", [
    (dict(dim=100), "heads * 64"), (dict(img_h=57), "multiples of 14"), (dict(ring_slots=0), "ring_slots"),
    (dict(batch=0), "batch"), (dict(depth=0), "depth"), (dict(mlp_kind=7), "mlp_kind"), (dict(dtype=3), "dtype"),
    (dict(weights_bytes=16), "weights_bytes"), (dict(ln_eps=0.0), "ln_eps"),
    (dict(taps=(C.c_int32 * 4)(1, 2, 2, 4)), "increasing"), (dict(depth=5), "taps[3]"),
])
def test_invalid_configurations_are_rejected_before_touching_the_device(over, needle):
    spec = vi.small_spec()
    blob = vi.pack_backbone(spec, vi.make_backbone_weights(spec, 1))
    c = _cfg(spec, blob, **over)
    with pytest.raises(vpe.VpeError) as ei:
        vpe.vpe_create(c, None, 0, None, 0)
    assert ei.value.code == vpe.VPE_EINVAL and needle in str(ei.value)
    with pytest.raises(vpe.VpeError):
        vpe.vpe_workspace_bytes(c, None, 0)


def test_invalid_heads_are_rejected():
    spec = vi.small_spec()
    blob = vi.pack_backbone(spec, vi.make_backbone_weights(spec, 1))
    c = _cfg(spec, blob)
    h = (vpe.binding.vpe_head_cfg * 1)()
    hb = vi.pack_head(spec, vi.HEAD_SEG, vi.make_head_weights(spec, vi.HEAD_SEG, 1))
    h[0].kind, h[0].classes, h[0].every_n, h[0].weights, h[0].weights_bytes = 0, spec.seg_classes, 0, hb.ctypes.data, hb.nbytes
    with pytest.raises(vpe.VpeError, match="every_n"):
        vpe.vpe_create(c, h, 1, None, 0)
    h[0].every_n, h[0].classes = 1, 300
    with pytest.raises(vpe.VpeError, match="classes"):
        vpe.vpe_create(c, h, 1, None, 0)
    h[0].classes, h[0].weights_bytes = spec.seg_classes, hb.nbytes - 4
    with pytest.raises(vpe.VpeError, match="weights_bytes"):
        vpe.vpe_create(c, h, 1, None, 0)


def test_workspace_bytes_accounts_for_ring_and_grows_with_slots():
    spec = vi.small_spec()
    blob = vi.pack_backbone(spec, vi.make_backbone_weights(spec, 1))
    a = vpe.vpe_workspace_bytes(_cfg(spec, blob, ring_slots=1), None, 0)
    b = vpe.vpe_workspace_bytes(_cfg(spec, blob, ring_slots=3), None, 0)
    slot = 4 * spec.batch * spec.tokens * spec.dim * 2
    assert b - a >= 2 * slot and b - a < 2 * slot + 8 * 256 * 2
    assert a > blob.nbytes // 2      # bf16 weights alone


def test_rate_divider_counts_are_exact_over_300_frames():
    # the paper's rate-limiting experiment (300 frames, several rates) made deterministic:
    # every_n = 1, 2, 3 must give exactly 300 / 150 / 100 executions
    eng, _, _ = make_engine(vi.small_spec(), 1, every_n=(1, 2, 3), flags=vpe.VPE_FLAG_HOST_ONLY)
    for f in range(300):
        fh = eng.encode(None)
        assert fh.frame == f and fh.slot == f % 2
        rcs = [eng.run_head(h, fh) for h in range(3)]
        assert rcs == [0, 0 if f % 2 == 0 else 1, 0 if f % 3 == 0 else 1]
    frames, runs, skips = eng.stats()
    assert frames == 300 and runs == [300, 150, 100] and skips == [0, 150, 200]


def test_rate_limits_in_hz_hold_within_one_frame_over_300_frames():
    # the paper's rate-limiting experiment (Appendix "Rate-Limiting Experiment" and its table: 300 images fed
    # at 30 Hz over 10 s, components limited to 5 / 10 / 15 / 20 / 25 / 30 Hz, ideal counts 50 .. 300, every
    # count within one frame of the ideal), with frame times as the clock; plus an odd rate, no limit, and a
    # limit above the input rate
    limits = [30.0, 15.0, 10.0, 20.0, 7.0, 0.0, 45.0, 5.0, 25.0]
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg",) * len(limits), flags=vpe.VPE_FLAG_HOST_ONLY)
    for h, hz in enumerate(limits):
        eng.set_head_rate_hz(h, hz)
    ran = [[] for _ in limits]
    for f in range(300):
        fh = eng.encode(None, t=f / 30.0)
        for h in range(len(limits)):
            if eng.run_head(h, fh) == 0:
                ran[h].append(f)
    for h, hz in enumerate(limits):
        want = 300 if hz == 0.0 or hz >= 30.0 else hz * 10.0
        assert abs(len(ran[h]) - want) <= 1, (hz, len(ran[h]))
        if 0.0 < hz < 30.0:
            gaps = np.diff(ran[h]) / 30.0
            # accumulating due times: single gaps may be one frame short of the period, never more, and any
            # two consecutive gaps together respect it
            assert gaps.min() >= 1.0 / hz - 1.0 / 30.0 - 1e-9
            assert gaps.max() <= 1.0 / hz + 1.0 / 30.0 + 1e-9
    assert ran[1] == list(range(0, 300, 2)) and ran[2] == list(range(0, 300, 3))
    assert ran[3][:5] == [0, 2, 3, 5, 6]                      # 20 Hz out of 30 Hz: two of every three frames
    assert [len(ran[h]) for h in (7, 2, 1, 3, 8, 0)] == [50, 100, 150, 200, 250, 300]     # the table's ideal counts
    frames, runs, skips = eng.stats()
    assert all(r + s == 300 for r, s in zip(runs, skips))


def test_rate_limit_in_hz_restarts_after_a_gap_and_combines_with_the_divider():
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg", "seg"), every_n=(1, 2), flags=vpe.VPE_FLAG_HOST_ONLY)
    eng.set_head_rate_hz(0, 10.0)
    eng.set_head_rate_hz(1, 10.0)
    times = [i / 100.0 for i in range(100)] + [6.0 + i / 100.0 for i in range(100)]     # 1 s, a 5 s pause, 1 s
    ran = [[], []]
    for t in times:
        fh = eng.encode(None, t=t)
        for h in range(2):
            if eng.run_head(h, fh) == 0:
                ran[h].append(t)
    for h in range(2):
        assert len(ran[h]) == 20                                  # 10 per second of input, no burst after the pause
        assert np.diff(ran[h]).min() >= 0.1 - 1e-9
        assert 6.0 in ran[h]                                      # the first frame after the pause runs at once
    # frames without a time are never limited in Hz; the limit can be lifted again
    fh = eng.encode(None)
    assert eng.run_head(0, fh) == 0
    eng.set_head_rate_hz(0, 0.0)
    for t in (7.0, 7.001, 7.002):
        assert eng.run_head(0, eng.encode(None, t=t)) == 0
    with pytest.raises(vpe.VpeError, match="backwards"):
        eng.encode(None, t=6.5)
    with pytest.raises(vpe.VpeError, match="max_hz"):
        eng.set_head_rate_hz(0, -1.0)
    with pytest.raises(vpe.VpeError, match="max_hz"):
        eng.set_head_rate_hz(0, float("nan"))
    with pytest.raises(vpe.VpeError, match="unknown head"):
        eng.set_head_rate_hz(5, 1.0)


def test_rate_can_change_at_run_time():
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg",), flags=vpe.VPE_FLAG_HOST_ONLY)
    ran = []
    for f in range(60):
        if f == 20:
            eng.set_head_rate(0, 5)
        if f == 40:
            eng.set_head_rate(0, 2)
        ran.append(eng.run_head(0, eng.encode(None)) == 0)
    expect = [True] * 20 + [f % 5 == 0 for f in range(20, 40)] + [f % 2 == 0 for f in range(40, 60)]
    assert ran == expect
    with pytest.raises(vpe.VpeError, match="every_n"):
        eng.set_head_rate(0, 0)
    with pytest.raises(vpe.VpeError, match="unknown head"):
        eng.set_head_rate(3, 1)


def test_latest_frame_policy_takes_the_newest_and_counts_what_it_passed_over():
    # the paper's decentralised modules (Sec. "Decentralization", "Data Flow"): a head that asks less often than
    # frames arrive works on the newest one; the frames in between are lost to it and counted; the ring, which
    # overwrites its oldest entry, reports the frames that left it without the head having asked
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg", "seg"), ring_slots=2, flags=vpe.VPE_FLAG_HOST_ONLY)
    assert eng.run_head_latest(0) == (vpe.VPE_SKIPPED, None)          # nothing encoded yet
    taken = []
    for f in range(20):
        fh = eng.encode(None)
        assert eng.run_head(1, fh) == 0                               # head 1 keeps pace, frame by frame
        if f % 5 == 4:                                                # head 0 asks after every 5th frame
            rc, got = eng.run_head_latest(0)
            assert rc == 0 and got.frame == f and got.slot == f % 2
            taken.append(got.frame)
            assert eng.run_head_latest(0) == (vpe.VPE_SKIPPED, None)  # same frame: nothing new
    assert taken == [4, 9, 14, 19]
    c0, c1 = eng.head_counters(0), eng.head_counters(1)
    assert c0["runs"] == 4 and c0["missed"] == 16 and c0["last_run_frame"] == 19 and c0["seen"] == 19
    # frames 0..17 were overwritten (2 slots): frame g leaves when frame g + 2 arrives, and counts for head 0
    # unless the head had by then asked about g or a later frame
    left_unasked = [g for g in range(18) if max([t for t in taken if t < g + 2], default=-1) < g]
    assert c0["overflow"] == len(left_unasked) == 12
    assert c1 == {"runs": 20, "skips": 0, "missed": 0, "overflow": 0, "busy": 0, "last_run_frame": 19, "seen": 19}
    frames, runs, skips = eng.stats()
    assert frames == 20 and runs == [4, 20] and skips == [0, 0]      # "nothing new" is not a rate skip


def test_latest_frame_policy_respects_the_divider_and_the_limit_in_hz():
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg", "seg"), every_n=(3, 1), ring_slots=3,
                            flags=vpe.VPE_FLAG_HOST_ONLY)
    eng.set_head_rate_hz(1, 10.0)
    ran = [[], []]
    for f in range(90):                                               # 30 Hz for 3 s, both heads ask every frame
        eng.encode(None, t=f / 30.0)
        for h in range(2):
            rc, got = eng.run_head_latest(h)
            if rc == 0:
                ran[h].append(got.frame)
    assert ran[0] == list(range(0, 90, 3))                            # at least 3 frames apart
    assert ran[1] == list(range(0, 90, 3))                            # 10 Hz out of 30 Hz
    for h in range(2):
        c = eng.head_counters(h)
        assert c["missed"] == 0 and c["overflow"] == 0 and c["runs"] == 30 and c["skips"] == 60
    # a head that asks only now and then still obeys its minimum distance, measured from its last run
    eng.set_head_rate(0, 4)
    got = []
    for f in range(90, 110):
        eng.encode(None, t=f / 30.0)
        if f % 3 == 0:
            rc, fh = eng.run_head_latest(0)
            if rc == 0:
                got.append(fh.frame)
    assert got == [93, 99, 105]                                       # asks at 90, 93, ...: 93 - 87 >= 4, then every 6
    f_new = eng.encode(None, t=4.0)
    assert eng.frame_ready(f_new) == vpe.VPE_OK                       # no device: complete at once
    assert eng.frame_ready(vpe.binding.vpe_feat(slot=(f_new.frame - 3) % 3, reserved=0, frame=f_new.frame - 3)) == vpe.VPE_ESTALE
    with pytest.raises(vpe.VpeError, match="not produced"):
        eng.frame_ready(vpe.binding.vpe_feat(slot=0, reserved=0, frame=1000))
    with pytest.raises(vpe.VpeError, match="unknown head"):
        eng.run_head_latest(2)
    with pytest.raises(vpe.VpeError, match="unknown head"):
        eng.head_counters(-1)


def test_wall_clock_engine_limits_in_real_time():
    import time
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg", "seg"), flags=vpe.VPE_FLAG_HOST_ONLY | vpe.VPE_FLAG_WALL_CLOCK)
    eng.set_head_rate_hz(0, 20.0)
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < 1.0:                             # about 1 s of frames every ~4 ms
        fh = eng.encode(None)
        eng.run_head(0, fh)
        eng.run_head(1, fh)
        n += 1
        time.sleep(0.004)
    span = time.perf_counter() - t0
    c0, c1 = eng.head_counters(0), eng.head_counters(1)
    assert c1["runs"] == n and n > 60
    assert abs(c0["runs"] - 20.0 * span) <= 2.5, (c0, span)           # one run of slack each for start and end
    # explicit times still work on such an engine, and must not run backwards against the clock
    with pytest.raises(vpe.VpeError, match="backwards"):
        eng.encode(None, t=0.0)


def test_ring_overwrites_oldest_and_stale_handles_are_refused():
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg",), ring_slots=2, flags=vpe.VPE_FLAG_HOST_ONLY)
    f0, f1 = eng.encode(None), eng.encode(None)
    assert (f0.slot, f1.slot) == (0, 1)
    assert eng.run_head(0, f0) == 0 and eng.run_head(0, f1) == 0      # both still resident
    f2 = eng.encode(None)                                            # reuses slot 0: frame 0 is gone
    assert f2.slot == 0
    with pytest.raises(vpe.VpeError) as ei:
        eng.run_head(0, f0)
    assert ei.value.code == vpe.VPE_ESTALE
    with pytest.raises(vpe.VpeError) as ei:
        vpe.vpe_feat_view(eng.handle, f0, 3)
    assert ei.value.code == vpe.VPE_ESTALE
    assert eng.run_head(0, f1) == 0 and eng.run_head(0, f2) == 0
    bogus = vpe.binding.vpe_feat(slot=1, reserved=0, frame=2)         # frame 2 lives in slot 0
    with pytest.raises(vpe.VpeError, match="not produced"):
        eng.run_head(0, bogus)
    future = vpe.binding.vpe_feat(slot=1, reserved=0, frame=7)
    with pytest.raises(vpe.VpeError, match="not produced"):
        eng.run_head(0, future)


def test_dpt_head_blob_size_and_validation():
    spec = vi.small_spec(head_ch=64)
    eng, _, hd = make_engine(spec, 1, kinds=("dpt", "seg"), flags=vpe.VPE_FLAG_HOST_ONLY)   # blob size accepted
    F = 64
    oc = [48, 96, 192, 384]
    assert hd[0]["up0_w"].shape == (48, 48, 4, 4) and hd[0]["down3_w"].shape == (384, 384, 3, 3)
    assert hd[0]["rn3_w"].shape == (F, 384, 3, 3) and hd[0]["head2_w"].shape == (32, 32, 3, 3)
    assert "fuse3_a_c1_w" not in hd[0] and "fuse2_a_c1_w" in hd[0]
    shape = vpe.vpe_head_output(eng.handle, 0, 0)[1]
    assert tuple(shape) == (1, spec.img_h, spec.img_w, 1)
    blob = vi.pack_backbone(spec, vi.make_backbone_weights(spec, 1))
    cfg = _cfg(spec, blob)
    hw = vi.pack_head(spec, vi.HEAD_DPT, hd[0])
    h = (vpe.binding.vpe_head_cfg * 1)()
    h[0].kind, h[0].classes, h[0].every_n, h[0].weights, h[0].weights_bytes = vi.HEAD_DPT, 0, 1, hw.ctypes.data, hw.nbytes
    for ch, needle in ((320, "64..256"), (96, "multiple of 64")):
        h[0].channels = ch
        with pytest.raises(vpe.VpeError, match=needle):
            vpe.vpe_workspace_bytes(cfg, h, 1)
    h[0].channels, h[0].weights_bytes = 64, hw.nbytes - 4
    with pytest.raises(vpe.VpeError, match="weights_bytes"):
        vpe.vpe_workspace_bytes(cfg, h, 1)
    h[0].weights_bytes = hw.nbytes
    assert vpe.vpe_workspace_bytes(cfg, h, 1) > hw.nbytes // 2


def test_feature_and_output_shapes():
    spec = vi.small_spec(registers=2, batch=2)
    eng, _, _ = make_engine(spec, 1, flags=vpe.VPE_FLAG_HOST_ONLY)
    fh = eng.encode(None)
    _, shape = vpe.vpe_feat_view(eng.handle, fh, 0)
    assert shape == (2, spec.tokens, spec.dim)
    assert vpe.vpe_head_output(eng.handle, 0, 0)[1] == (2, spec.gh, spec.gw, spec.seg_classes)
    assert vpe.vpe_head_output(eng.handle, 0, 1)[1] == (2, spec.img_h, spec.img_w, 1)
    assert vpe.vpe_head_output(eng.handle, 1, 0)[1] == (2, spec.img_h, spec.img_w, 1)
    assert vpe.vpe_head_output(eng.handle, 2, 0)[1] == (2, spec.gh, spec.gw, spec.det_classes + 4)
    assert vpe.vpe_head_output(eng.handle, 2, 1)[1] == (2, spec.gh, spec.gw, 1)
    with pytest.raises(vpe.VpeError):
        vpe.vpe_head_output(eng.handle, 1, 1)


def test_create_without_a_device_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(vpe.VpeError) as ei:
        make_engine(vi.small_spec(), 1, kinds=("seg",), torch_workspace=False)
    assert ei.value.code in (vpe.VPE_ENOMEM, vpe.VPE_EHIP)


def test_next_encode_stream_is_null_without_a_device():
    eng, _, _ = make_engine(vi.small_spec(), 1, kinds=("seg",), flags=vpe.VPE_FLAG_HOST_ONLY)
    assert eng.next_encode_stream() is None


def test_preprocess_rejects_bad_arguments_before_touching_the_device():
    ok = dict(frames_ptr=4096, batch=1, src_h=8, src_w=8, images_ptr=8192, dst_h=4, dst_w=4, mean=(0, 0, 0), std=(1, 1, 1))
    for over, needle in [(dict(frames_ptr=None), "null"), (dict(images_ptr=None), "null"), (dict(batch=0), "positive"),
                         (dict(src_w=0), "positive"), (dict(dst_h=-3), "positive"), (dict(std=(1, 0, 1)), "std"),
                         (dict(std=(1, 1, float("nan"))), "std"), (dict(mean=(float("inf"), 0, 0)), "mean"),
                         (dict(src_h=40000, src_w=40000), "too large")]:
        with pytest.raises(vpe.VpeError, match=needle):
            vpe.vpe_preprocess_u8(**{**ok, **over})


def test_head_completion_and_stage_times_without_a_device():
    eng, _, _ = make_engine(vi.small_spec(), 1, flags=vpe.VPE_FLAG_HOST_ONLY | vpe.VPE_FLAG_TIMING)
    assert eng.head_done(0)                                     # never ran: nothing to wait for
    fh = eng.encode(None)
    assert eng.run_head(1, fh) == vpe.VPE_OK
    assert eng.head_done(1)
    eng.wait_head(1)
    assert eng.stage_times() == (-1.0, [-1.0, -1.0, -1.0])      # no device, no figures
    with pytest.raises(vpe.VpeError):
        vpe.vpe_head_done(eng.handle, 3)
    plain, _, _ = make_engine(vi.small_spec(), 1, flags=vpe.VPE_FLAG_HOST_ONLY)
    with pytest.raises(vpe.VpeError, match="VPE_FLAG_TIMING"):
        plain.stage_times()


def test_static_scratch_head_run_checks_sizes_on_the_host():
    # vpe_run_head_static refuses heads whose intermediate buffers exceed the library's 8 MiB static array
    spec = vi.CONFIGS["cfg2"]
    w = vi.make_backbone_weights(spec, 1)
    eng, _, _ = make_engine(spec, 1, kinds=("seg", "depth", "det", "dpt"), flags=vpe.VPE_FLAG_HOST_ONLY, weights=w)
    fh = eng.encode(None)
    assert vpe.vpe_run_head_static(eng.handle, 0, fh) == vpe.VPE_OK
    assert vpe.vpe_run_head_static(eng.handle, 2, fh) == vpe.VPE_OK          # 1530 x 512 bf16 = 1.6 MB
    with pytest.raises(vpe.VpeError, match="needs 10[0-9]{7} bytes of scratch, the static array holds 8388608"):
        vpe.vpe_run_head_static(eng.handle, 1, fh)
    with pytest.raises(vpe.VpeError, match="DPT"):
        vpe.vpe_run_head_static(eng.handle, 3, fh)
    with pytest.raises(vpe.VpeError):
        vpe.vpe_run_head_static(eng.handle, 4, fh)
    assert eng.stats()[1] == [1, 0, 1, 0]
