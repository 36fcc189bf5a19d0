"""GPU checks of the engine's sharing and scheduling properties (paper, Sec. "System architecture"):
features are written once and read in place, slots are reused safely, rates hold on the device,
graph replay equals eager launches bit for bit, and nothing allocates after create."""
import numpy as np
import pytest
import torch

import paper_2508_11584_amd as vpe
import vpe_inputs as vi
from helpers import make_engine

pytestmark = pytest.mark.gpu

SPEC = vi.ModelSpec("engine", dim=128, depth=4, heads=2, mlp_hidden=256, img_h=98, img_w=154, taps=(1, 2, 3, 4),
                    head_ch=64, dtype="bf16")


def outputs(eng):
    return [eng.head_output(0, 0).clone(), eng.head_output(0, 1).clone(), eng.head_output(1, 0).clone(),
            eng.head_output(2, 0).clone(), eng.head_output(2, 1).clone()]


def frames(n, seed=300):
    return [torch.from_numpy(vi.make_batch(SPEC, seed + i)).cuda() for i in range(n)]


def test_heads_read_the_slot_in_place_and_leave_it_untouched():
    eng, _, _ = make_engine(SPEC, 11)
    img = frames(1)[0]
    fh = eng.encode(img)
    eng.sync()
    before = [eng.feat_view(fh, k).clone() for k in range(4)]
    ptrs = [eng.feat_ptr(fh, k) for k in range(4)]
    for h in range(3):
        assert eng.run_head(h, fh) == 0
    eng.sync()
    assert [eng.feat_ptr(fh, k) for k in range(4)] == ptrs            # same device memory, no copy made
    for k in range(4):
        assert torch.equal(eng.feat_view(fh, k), before[k])
    # the four maps of a slot are distinct regions inside the engine's single workspace
    assert len(set(ptrs)) == 4
    lo = eng._ws.data_ptr()
    assert all(lo <= p < lo + eng._ws.numel() for p in ptrs)
    eng.close()


def test_graph_replay_equals_eager_bit_for_bit_over_several_frames():
    fs = frames(5)
    res = {}
    for flags in (0, vpe.VPE_FLAG_GRAPHS):
        eng, _, _ = make_engine(SPEC, 12, flags=flags)
        per_frame = []
        for f in fs:                       # replays interleaved with syncs and host reads
            fh = eng.encode(f)
            for h in range(3):
                eng.run_head(h, fh)
            eng.sync()
            per_frame.append([eng.feat_view(fh, 3).clone()] + outputs(eng))
        res[flags] = per_frame
        eng.close()
    for a, b in zip(res[0], res[vpe.VPE_FLAG_GRAPHS]):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
    # different frames really give different results (the replay is not returning a stale buffer)
    assert not torch.equal(res[0][0][0], res[0][1][0])


def test_shared_path_equals_sequential_recompute_bit_for_bit():
    eng, _, _ = make_engine(SPEC, 13, flags=vpe.VPE_FLAG_GRAPHS)
    img = frames(1)[0]
    fh = eng.encode(img)
    for h in range(3):
        eng.run_head(h, fh)
    eng.sync()
    shared = outputs(eng)
    one = torch.cuda.Stream()
    seq = []
    for h in range(3):                      # every head recomputes its own backbone pass, one stream
        fh = eng.encode(img, stream=one)
        eng.run_head(h, fh, stream=one)
        eng.sync()
        seq.append(outputs(eng))
    final = [seq[0][0], seq[0][1], seq[1][2], seq[2][3], seq[2][4]]
    for a, b in zip(shared, final):
        assert torch.equal(a, b)
    eng.close()


def test_single_slot_ring_and_back_to_back_frames_stay_correct():
    # slot recycling with 1, 2 and 3 slots (graphs captured per slot) gives the same per-frame results
    fs = frames(6, seed=400)
    ref = []
    eng, _, _ = make_engine(SPEC, 14, ring_slots=2)
    for f in fs:
        fh = eng.encode(f)
        for h in range(3):
            eng.run_head(h, fh)
        eng.sync()
        ref.append(outputs(eng))
    eng.close()
    for slots in (1, 2, 3):
        eng, _, _ = make_engine(SPEC, 14, ring_slots=slots, flags=vpe.VPE_FLAG_GRAPHS)
        got = []
        for f in fs:
            fh = eng.encode(f)
            for h in range(3):
                eng.run_head(h, fh)
            eng.sync()                      # head outputs are single-instance: read them before the next frame
            got.append(outputs(eng))
        for a, b in zip(ref, got):
            for x, y in zip(a, b):
                assert torch.equal(x, y)
        eng.close()


@pytest.mark.parametrize("lanes,slots,head_streams", [(1, 2, 0), (2, 2, 0), (2, 3, 0), (2, 3, 1), (3, 4, 2), (4, 4, 3)])
def test_unsynchronised_stream_of_frames_ends_in_the_right_state(lanes, slots, head_streams):
    # 40 frames pushed without any host sync, rates 1/2/3, one to four encoder lanes (the encoder passes of
    # consecutive frames overlap) and heads on own or shared streams: the final outputs must be those of
    # the last frame each head was due on, computed in isolation
    fs = frames(4, seed=500)
    eng, _, _ = make_engine(SPEC, 15, every_n=(1, 2, 3), flags=vpe.VPE_FLAG_GRAPHS, ring_slots=slots,
                            encoder_lanes=lanes, head_streams=head_streams)
    n = 40
    for i in range(n):
        fh = eng.encode(fs[i % 4])
        for h in range(3):
            eng.run_head(h, fh)
    eng.sync()
    got = outputs(eng)
    frames_done, runs, skips = eng.stats()
    assert frames_done == n and runs == [40, 20, 14] and skips == [0, 20, 26]
    eng.close()
    last_due = [39, 38, 39]                  # last frame index with f % every_n == 0, for every_n = 1, 2, 3
    eng, _, _ = make_engine(SPEC, 15)
    exp = {}
    for h, f in enumerate(last_due):
        fh = eng.encode(fs[f % 4])
        eng.run_head(h, fh)
        eng.sync()
        exp[h] = outputs(eng)
    want = [exp[0][0], exp[0][1], exp[1][2], exp[2][3], exp[2][4]]
    for a, b in zip(got, want):
        assert torch.equal(a, b)
    eng.close()


def test_no_device_allocation_after_create():
    eng, _, _ = make_engine(SPEC, 16, flags=vpe.VPE_FLAG_GRAPHS)
    fs = frames(2)
    for i in range(4):                       # warm-up captures the graphs
        fh = eng.encode(fs[i % 2])
        for h in range(3):
            eng.run_head(h, fh)
    eng.sync()
    free0, _ = torch.cuda.mem_get_info()
    for i in range(300):
        fh = eng.encode(fs[i % 2])
        for h in range(3):
            eng.run_head(h, fh)
    eng.sync()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0                    # driver-level free memory unchanged over 300 frames
    eng.close()


def test_library_owned_workspace_works_without_torch_memory():
    eng, _, _ = make_engine(SPEC, 17, torch_workspace=False)
    eng2, _, _ = make_engine(SPEC, 17)
    img = frames(1)[0]
    for e in (eng, eng2):
        fh = e.encode(img)
        for h in range(3):
            e.run_head(h, fh)
        e.sync()
    for a, b in zip(outputs(eng), outputs(eng2)):
        assert torch.equal(a, b)
    eng.close()
    eng2.close()


def test_batch_elements_are_independent_on_the_device():
    spec = vi.with_(SPEC, batch=3)
    eng, _, _ = make_engine(spec, 18)
    imgs = vi.make_batch(spec, 600)
    fh = eng.encode(torch.from_numpy(imgs).cuda())
    for h in range(3):
        eng.run_head(h, fh)
    eng.sync()
    batched = [eng.feat_view(fh, 3).clone(), eng.head_output(1, 0).clone(), eng.head_output(2, 0).clone()]
    eng.close()
    eng1, _, _ = make_engine(SPEC, 18)
    for b in range(3):
        fh = eng1.encode(torch.from_numpy(imgs[b:b + 1]).cuda())
        for h in range(3):
            eng1.run_head(h, fh)
        eng1.sync()
        assert torch.equal(eng1.feat_view(fh, 3)[0], batched[0][b])
        assert torch.equal(eng1.head_output(1, 0)[0], batched[1][b])
        assert torch.equal(eng1.head_output(2, 0)[0], batched[2][b])
    eng1.close()


def test_encoder_lanes_and_shared_head_streams_give_the_same_frames_as_one_lane():
    fs = frames(6, seed=700)
    res = {}
    for lanes, slots, hs in ((1, 2, 0), (2, 2, 0), (3, 3, 1)):
        eng, _, _ = make_engine(SPEC, 19, flags=vpe.VPE_FLAG_GRAPHS, ring_slots=slots, encoder_lanes=lanes, head_streams=hs)
        feats = []
        handles = []
        for f in fs[:2]:                          # two frames in flight before anything is read
            handles.append(eng.encode(f))
        eng.sync()
        feats += [eng.feat_view(h, 3).clone() for h in handles]
        for f in fs[2:]:
            fh = eng.encode(f)
            for h in range(3):
                eng.run_head(h, fh)
            eng.sync()
            feats.append(eng.feat_view(fh, 3).clone())
            feats += outputs(eng)
        res[lanes] = feats
        eng.close()
    for other in (2, 3):
        for a, b in zip(res[1], res[other]):
            assert torch.equal(a, b)


def test_rate_limit_in_hz_on_the_device():
    # 12 frames stamped at 30 Hz, depth limited to 15 Hz and detection to 10 Hz: the outputs left at the end
    # are those of the last frame each head was allowed to run on (seg 11, depth 10, det 9)
    fs = frames(4, seed=900)
    eng, _, _ = make_engine(SPEC, 21, flags=vpe.VPE_FLAG_GRAPHS, ring_slots=3, encoder_lanes=2)
    eng.set_head_rate_hz(1, 15.0)
    eng.set_head_rate_hz(2, 10.0)
    ran = {0: [], 1: [], 2: []}
    for i in range(12):
        fh = eng.encode(fs[i % 4], t=i / 30.0)
        for h in range(3):
            if eng.run_head(h, fh) == 0:
                ran[h].append(i)
    eng.sync()
    got = outputs(eng)
    eng.close()
    assert ran == {0: list(range(12)), 1: [0, 2, 4, 6, 8, 10], 2: [0, 3, 6, 9]}
    eng, _, _ = make_engine(SPEC, 21)
    exp = {}
    for h in range(3):
        fh = eng.encode(fs[ran[h][-1] % 4])
        eng.run_head(h, fh)
        eng.sync()
        exp[h] = outputs(eng)
    for a, b in zip(got, [exp[0][0], exp[0][1], exp[1][2], exp[2][3], exp[2][4]]):
        assert torch.equal(a, b)
    eng.close()


def test_newest_frame_policy_on_the_device_never_queues_behind_a_running_head():
    # a producer that stays at most one ring ahead of the device, every head asking for the newest complete frame
    # after each: a call starts the head, is turned away because the previous run is still going, or finds no
    # complete new frame; what a head holds at the end is the result of the last frame it reported, computed alone
    fs = frames(4, seed=1000)
    eng, _, _ = make_engine(SPEC, 22, flags=vpe.VPE_FLAG_GRAPHS, ring_slots=3, encoder_lanes=2)
    n = 60
    handles = []
    ran = {0: [], 1: [], 2: []}

    def poll():
        for h in range(3):
            rc, fh = eng.run_head_latest(h)
            assert rc in (vpe.VPE_OK, vpe.VPE_BUSY, vpe.VPE_SKIPPED)
            if rc == vpe.VPE_OK:
                assert eng.frame_ready(fh) == vpe.VPE_OK
                ran[h].append(fh.frame)

    for i in range(n):
        while i >= 2 and eng.frame_ready(handles[i - 2]) == vpe.VPE_BUSY:
            poll()
        handles.append(eng.encode(fs[i % 4]))
        poll()
    eng.sync()
    assert eng.frame_ready(handles[-1]) == vpe.VPE_OK and eng.frame_ready(handles[0]) == vpe.VPE_ESTALE
    poll()                                                             # idle now: every head takes frame n - 1 unless it has it
    eng.sync()
    got = outputs(eng)
    for h in range(3):
        c = eng.head_counters(h)
        assert ran[h] == sorted(set(ran[h])) and ran[h][-1] == n - 1 and len(ran[h]) >= 2
        assert c["runs"] == len(ran[h]) and c["skips"] == 0
        assert c["last_run_frame"] == c["seen"] == n - 1
        assert c["missed"] == n - c["runs"]                        # every frame either ran or was passed over
    eng.close()
    eng, _, _ = make_engine(SPEC, 22)
    fh = eng.encode(fs[(n - 1) % 4])
    for h in range(3):
        eng.run_head(h, fh)
    eng.sync()
    for a, b in zip(got, outputs(eng)):
        assert torch.equal(a, b)
    eng.close()


def test_head_completion_query_and_stage_times():
    # a consumer takes a head's result without waiting for the rest of the engine (paper, Sec. "Head Module":
    # results go to the head's output buffer; Sec. "Decentralization": nobody blocks on anybody)
    eng, _, _ = make_engine(SPEC, 11, flags=vpe.VPE_FLAG_TIMING, ring_slots=2)
    assert eng.head_done(1) and eng.stage_times() == (-1.0, [-1.0, -1.0, -1.0])
    fr = frames(2)
    fh = eng.encode(fr[0])
    for h in range(3):
        assert eng.run_head(h, fh) == 0
    eng.wait_head(0)                                             # seg only; depth may still be running
    assert eng.head_done(0)
    seg = eng.head_output(0, 1).clone()
    eng.sync()
    assert all(eng.head_done(h) for h in range(3))
    enc_ms, head_ms = eng.stage_times()
    assert 0.0 < enc_ms < 50.0 and all(0.0 < t < 50.0 for t in head_ms), (enc_ms, head_ms)
    # a second frame with only the depth head: the seg head's output buffer keeps its result
    fh = eng.encode(fr[1])
    assert eng.run_head(1, fh) == 0
    eng.sync()
    assert torch.equal(eng.head_output(0, 1), seg)
    eng.close()


def test_sync_waits_for_work_on_caller_streams_too():
    eng, _, _ = make_engine(SPEC, 11)
    st = torch.cuda.Stream()
    img = frames(1)[0]
    fh = eng.encode(img, stream=st)
    for h in range(3):
        eng.run_head(h, fh, stream=st)
    eng.sync()                                                   # engine events, not a device-wide wait
    assert st.query()
    ref = outputs(eng)
    fh = eng.encode(img)
    for h in range(3):
        eng.run_head(h, fh)
    eng.sync()
    for a, b in zip(ref, outputs(eng)):
        assert torch.equal(a, b)
    eng.close()
