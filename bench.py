"""Benchmark of the hot path on one MI355X: ViT-S/14 bf16 at 476x630 with three heads.

One step = one frame through the whole path: vpe_encode (backbone, written once into the
shared feature slot) + the seg, depth and det heads reading that slot in place on their own
streams.  Inputs are synthetic and already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch of the dominant kernel as the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes measured
    them (calibrated against a 1 GiB copy): the `traffic_bytes_per_launch:` line of the tracked summary
    profiles/<kernel>_<workload>_hbm_traffic.txt, or None when no such pass has been taken for this workload."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.strip().startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def backbone_flops(spec) -> float:
    """Algorithmic FLOP of one encoder pass: patch embedding + per block QKV, attention (4 N^2 D,
    no causal discount), out-projection and MLP.  LayerNorm / activation work is not counted."""
    B, P, N, D, T = spec.batch, spec.patches, spec.tokens, spec.dim, spec.batch * spec.tokens
    per_block = 2.0 * T * D * 3 * D + 4.0 * B * N * N * D + 2.0 * T * D * D + 2.0 * T * D * spec.fc1_out \
        + 2.0 * T * spec.mlp_hidden * D
    return 2.0 * B * P * 588 * D + spec.depth * per_block


class RawStream:
    """A HIP stream by handle, in the shape the Engine wrapper expects of a stream argument."""
    def __init__(self, handle: int):
        self.cuda_stream = handle


def make_masked_streams(vpe, k: int):
    """k streams, stream i restricted to compute units [i * 256 / k, (i + 1) * 256 / k) by a CU mask; [] if the
    runtime refuses.  The runtime call is taken from the HIP library that libvpe.so is linked against."""
    import ctypes as C
    try:
        create = vpe.lib().hipExtStreamCreateWithCUMask
    except AttributeError:
        return []
    create.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint32)]
    create.restype = C.c_int
    out, per = [], 256 // k
    for i in range(k):
        words = (C.c_uint32 * 8)()
        for cu in range(i * per, (i + 1) * per):
            words[cu // 32] |= 1 << (cu % 32)
        h = C.c_void_p()
        if create(C.byref(h), 8, words) != 0 or not h.value:
            destroy_streams(vpe, out)
            return []
        out.append(RawStream(h.value))
    return out


def destroy_streams(vpe, streams) -> None:
    import ctypes as C
    if not streams:
        return
    destroy = vpe.lib().hipStreamDestroy
    destroy.argtypes = [C.c_void_p]
    destroy.restype = C.c_int
    for st in streams:
        destroy(st.cuda_stream)


def multihead_experiment(args, vpe, vi, make_engine, np, torch) -> None:
    """Frame latency (submit one resident frame, wait for every head) against the number k of identical heads.

    Arms, all on the same engine and kernels (paper, Sec. "Single Backbone vs. Independent Models" and
    "Parallel vs. Sequential Processing"):
      independent       k x (encoder pass + head) one after another on one stream: k separate full models
      sequential_heads  one encoder pass, then the k heads one after another on that stream
      concurrent        one encoder pass, the k heads spread over the engine's head streams
      concurrent_cu_masked  one encoder pass, every head on a stream of its own that may use 256 / k compute units
    plus the pipelined rate of the concurrent arm (frames/s without waiting between frames, several encoder
    lanes) and the device memory each added head costs."""
    spec = vi.CONFIGS[args.config]
    wseed, iseed = vi.SEEDS[args.config]
    images_np = vi.make_batch(spec, iseed)
    frames = [torch.from_numpy(images_np).cuda(), torch.from_numpy(np.ascontiguousarray(images_np[..., ::-1])).cuda()]
    one = torch.cuda.Stream()
    n = max(10, min(args.steps, 60))
    rows = []
    for kind in ("depth", "det"):
        base_ws = None
        for k in (1, 2, 4, 8):
            eng, _, _ = make_engine(spec, wseed, kinds=(kind,) * k, ring_slots=2, flags=0 if args.no_graphs else vpe.VPE_FLAG_GRAPHS)

            def independent(i):
                for h in range(k):
                    fh = eng.encode(frames[i & 1], stream=one)
                    eng.run_head(h, fh, stream=one)

            def sequential_heads(i):
                fh = eng.encode(frames[i & 1], stream=one)
                for h in range(k):
                    eng.run_head(h, fh, stream=one)

            def concurrent(i):
                fh = eng.encode(frames[i & 1])
                for h in range(k):
                    eng.run_head(h, fh)

            # the same with every head on its own stream restricted to 256 / k compute units (a CU mask; the
            # analogue of the fixed GPU shares the paper gives its head processes through MPS)
            masked = make_masked_streams(vpe, k)

            def concurrent_masked(i):
                fh = eng.encode(frames[i & 1])
                for h in range(k):
                    eng.run_head(h, fh, stream=masked[h])

            def latency(fn):
                lat = []
                for i in range(n + 5):
                    t0 = time.perf_counter()
                    fn(i)
                    eng.sync()
                    lat.append((time.perf_counter() - t0) * 1e3)
                lat = sorted(lat[5:])
                return lat[len(lat) // 2]

            row = {"head": kind, "k": k, "independent_ms": round(latency(independent), 4),
                   "sequential_heads_ms": round(latency(sequential_heads), 4), "concurrent_ms": round(latency(concurrent), 4),
                   "workspace_mb": round(eng.workspace_bytes / 1e6, 1)}
            row["concurrent_cu_masked_ms"] = round(latency(concurrent_masked), 4) if masked else None
            eng.sync()
            destroy_streams(vpe, masked)
            eng.close()
            # pipelined rate: frames are pushed without waiting, consecutive encoder passes overlap
            lanes = args.encoder_lanes or 3
            eng, _, _ = make_engine(spec, wseed, kinds=(kind,) * k, ring_slots=lanes + 1, encoder_lanes=lanes,
                                    flags=0 if args.no_graphs else vpe.VPE_FLAG_GRAPHS)
            for i in range(10):
                concurrent(i)
            eng.sync()
            t0 = time.perf_counter()
            for i in range(n):
                concurrent(i)
            eng.sync()
            row["concurrent_pipelined_fps"] = round(n * spec.batch / (time.perf_counter() - t0), 1)
            eng.close()
            row["independent_over_concurrent"] = round(row["independent_ms"] / row["concurrent_ms"], 3)
            row["sequential_over_concurrent"] = round(row["sequential_heads_ms"] / row["concurrent_ms"], 3)
            if base_ws is None:
                base_ws = row["workspace_mb"]
            row["mb_per_added_head"] = round((row["workspace_mb"] - base_ws) / (k - 1), 1) if k > 1 else None
            rows.append(row)
            print(json.dumps(row), file=sys.stderr, flush=True)
    print(json.dumps({"experiment": "multihead", "workload": spec.name, "frames_per_point": n, "hw_queues": args.hw_queues,
                      "latency": "median ms, one frame at a time, inputs resident in HBM", "rows": rows}))


def freshness_experiment(args, vpe, vi, make_engine, np, torch) -> None:
    """The lossy, decentralised way of running the engine (paper, Sec. "Decentralization", "Data Flow", "Dynamic
    Frequency Control", Appendix "Rate-Limiting Experiment"), on the host's real clock.

    rate_limit: 300 frames published at a fixed rate, every head limited to the same rate in Hz, engine
      stamping frames with its own steady clock; delivered counts against rate x duration (the appendix's table;
      its 30 Hz / 10 s stream is run ten times faster here, 300 Hz / 1 s, limits 50 .. 300 Hz).
    saturated: frames pushed as fast as the encoder takes them (the producer stays one encode per lane ahead of
      the device) while every head keeps asking for the newest complete frame and is turned away while its previous
      run is still going: nothing waits for anything else, slow heads lose frames."""
    spec = vi.CONFIGS[args.config]
    wseed, iseed = vi.SEEDS[args.config]
    kinds = ("seg", "depth", "det")
    images_np = vi.make_batch(spec, iseed)
    frames = [torch.from_numpy(images_np).cuda(), torch.from_numpy(np.ascontiguousarray(images_np[..., ::-1])).cuda()]
    flags = (0 if args.no_graphs else vpe.VPE_FLAG_GRAPHS) | vpe.VPE_FLAG_WALL_CLOCK
    lanes = args.encoder_lanes
    publish_hz, n = 300.0, 300
    table = []
    for limit in (50.0, 100.0, 150.0, 200.0, 250.0, 300.0):
        eng, _, _ = make_engine(spec, wseed, kinds=kinds, ring_slots=lanes + 1, encoder_lanes=lanes, flags=flags)
        for i in range(6):                                    # graph capture, not limited
            fh = eng.encode(frames[i & 1])
            for h in range(3):
                eng.run_head(h, fh)
        eng.sync()
        before = [eng.head_counters(h)["runs"] for h in range(3)]
        for h in range(3):
            eng.set_head_rate_hz(h, limit)
        t0 = time.perf_counter()
        for i in range(n):
            while time.perf_counter() - t0 < i / publish_hz:
                pass
            fh = eng.encode(frames[i & 1])
            for h in range(3):
                eng.run_head(h, fh)
        eng.sync()
        span = time.perf_counter() - t0
        got = [eng.head_counters(h)["runs"] - before[h] for h in range(3)]
        ideal = n * limit / publish_hz
        table.append({"limit_hz": limit, "ideal": ideal, "delivered": dict(zip(kinds, got)),
                      "error": dict(zip(kinds, [g - ideal for g in got])), "span_s": round(span, 4)})
        eng.close()
        print(json.dumps(table[-1]), file=sys.stderr, flush=True)
    eng, _, _ = make_engine(spec, wseed, kinds=kinds, ring_slots=lanes + 1, encoder_lanes=lanes, flags=flags)
    for i in range(6):
        fh = eng.encode(frames[i & 1])
        for h in range(3):
            eng.run_head(h, fh)
    eng.sync()
    c0 = [eng.head_counters(h) for h in range(3)]
    n_sat = max(args.steps, 300) * 4
    pending = []

    def poll():
        for h in range(3):
            eng.run_head_latest(h)

    t0 = time.perf_counter()
    for i in range(n_sat):
        while len(pending) >= lanes and eng.frame_ready(pending[0]) == vpe.VPE_BUSY:     # stay `lanes` encodes ahead at most
            poll()
        if len(pending) >= lanes:
            pending.pop(0)
        pending.append(eng.encode(frames[i & 1]))
        poll()
    eng.sync()
    span = time.perf_counter() - t0
    heads = {}
    for h, kind in enumerate(kinds):
        c = eng.head_counters(h)
        runs = c["runs"] - c0[h]["runs"]
        heads[kind] = {"runs": runs, "runs_per_s": round(runs / span, 1), "missed": c["missed"] - c0[h]["missed"],
                       "busy_returns": c["busy"] - c0[h]["busy"], "overflow": c["overflow"] - c0[h]["overflow"]}
    eng.close()
    print(json.dumps({"experiment": "freshness", "workload": spec.name, "encoder_lanes": lanes, "hw_queues": args.hw_queues,
                      "rate_limit": {"published_hz": publish_hz, "frames": n, "rows": table},
                      "saturated": {"frames": n_sat, "encoder_frames_per_s": round(n_sat * spec.batch / span, 1), "heads": heads}}))


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="cfg2", help="cfg1..cfg5 (cfg2 is the headline workload)")
    ap.add_argument("--no-graphs", action="store_true")
    ap.add_argument("--encoder-lanes", type=int, default=None,
                    help="k = the encoder passes of k consecutive frames overlap on the GPU (throughput pipelining); "
                         "default 3 for the one-image configs 1-3, 2 for the batched configs 4-5")
    ap.add_argument("--ring-slots", type=int, default=None, help="feature ring size; default encoder lanes + 1")
    ap.add_argument("--hw-queues", type=int, default=5,
                    help="hardware queues the HIP runtime may use in this process (GPU_MAX_HW_QUEUES; the default "
                         "stream keeps one, the engine's lanes + head streams want four); 0 = leave the environment alone")
    ap.add_argument("--heads", default=None,
                    help="comma-separated head kinds in place of the workload's own (seg,depth,det): e.g. seg,dpt,det runs "
                         "the full DPT depth head (--head-ch sets its width); not the headline workload")
    ap.add_argument("--head-ch", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=50)
    ap.add_argument("--roofline-only", action="store_true",
                    help="one frame, a 1 GiB device copy (counter calibration) and the dominant-kernel timing leg only; "
                         "the mode the rocprofv3 --pmc passes are taken in")
    ap.add_argument("--kernel-pass", action="store_true",
                    help="one frame, then every kernel family of the timing aid alone (1 + --kernel-reps launches each): "
                         "the mode the per-kernel rocprofv3 --pmc passes are taken in")
    ap.add_argument("--experiment", choices=["multihead", "freshness"], default=None,
                    help="multihead: frame latency against the number of identical heads (1, 2, 4, 8), for depth heads "
                         "(the paper's single-backbone-vs-independent-models experiment) and detection heads (its "
                         "parallel-vs-sequential-heads experiment); freshness: the appendix's rate-limiting table on the real "
                         "clock, and the lossy newest-frame policy under a saturating producer; each prints its own JSON "
                         "line instead of the benchmark's")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch of the dominant kernel from the --pmc passes (FETCH_SIZE + WRITE_SIZE, "
                         "calibrated); reported as roofline.traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); use --gpus 1")
    if args.hw_queues > 0:
        os.environ["GPU_MAX_HW_QUEUES"] = str(args.hw_queues)      # read by the runtime when it initialises (below)
    if args.encoder_lanes is None:
        args.encoder_lanes = 3 if args.config in ("cfg1", "cfg2", "cfg3") else 2
    if args.ring_slots is None:
        args.ring_slots = args.encoder_lanes + 1

    import numpy as np
    import torch

    import paper_2508_11584_amd as vpe
    import vpe_inputs as vi
    from paper_2508_11584_amd.synthetic import make_engine

    if args.experiment == "multihead":
        multihead_experiment(args, vpe, vi, make_engine, np, torch)
        return
    if args.experiment == "freshness":
        freshness_experiment(args, vpe, vi, make_engine, np, torch)
        return

    spec = vi.CONFIGS[args.config]
    wseed, iseed = vi.SEEDS[args.config]
    kinds = ("seg",) if args.config == "cfg1" else ("seg", "depth", "det")
    if args.heads:
        kinds = tuple(args.heads.split(","))
    if args.head_ch:
        spec = vi.with_(spec, head_ch=args.head_ch)
    flags = 0 if args.no_graphs else vpe.VPE_FLAG_GRAPHS
    eng, w, hw = make_engine(spec, wseed, kinds=kinds, ring_slots=args.ring_slots, flags=flags, encoder_lanes=args.encoder_lanes)
    head_streams = min(len(kinds), max(1, 4 - args.encoder_lanes))      # the engine's rule (include/vpe.h, head_streams = 0)
    images_np = vi.make_batch(spec, iseed)
    # two distinct resident frames, alternated, so no step can reuse the previous step's result
    frames = [torch.from_numpy(images_np).cuda(), torch.from_numpy(np.ascontiguousarray(images_np[..., ::-1])).cuda()]
    nh = len(kinds)

    def shared_step(i):
        fh = eng.encode(frames[i & 1])
        for h in range(nh):
            eng.run_head(h, fh)

    one = torch.cuda.Stream()

    def sequential_step(i):
        # baseline: every head recomputes its own backbone pass, all on one stream
        for h in range(nh):
            fh = eng.encode(frames[i & 1], stream=one)
            eng.run_head(h, fh, stream=one)

    def independent_pipelined_step(i):
        # the same baseline given everything the shared path gets -- the engine's encoder lanes, head streams,
        # ring and hardware queues: one encoder pass per head, consecutive passes overlapping on the lanes
        for h in range(nh):
            fh = eng.encode(frames[i & 1])
            eng.run_head(h, fh)

    def encode_step(i):
        eng.encode(frames[i & 1])

    def bracketed(fn, steps):
        """Seconds for `steps` steps between two synchronisations (pipeline fill and drain included)."""
        eng.sync()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        eng.sync()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def timed(fn, steps, warmup):
        """Seconds per step in steady state.  A run of n steps between two synchronisations costs the steady
        time of n steps plus one fill-and-drain of the pipeline (about one frame latency, whatever n is); timing
        `prime + steps` steps and `prime` steps and taking the difference leaves exactly `steps` steady-state
        steps, so a short run and a long run report the same rate.  Returns (steady, bracketed) seconds per step,
        the second being the plain synchronise / steps / synchronise figure."""
        for i in range(warmup):
            fn(i)
        prime = 2 * args.encoder_lanes + 2
        short = sorted(bracketed(fn, prime) for _ in range(5))[2]
        long_ = bracketed(fn, prime + steps)
        return (long_ - short) / steps, bracketed(fn, steps) / steps

    def settled_kernel_time(which):
        # A kernel launched in a row behind lighter work first runs at the clock that work left behind: the dominant
        # convolution takes 116, 109, 102, 99, 98 us per launch over its first five batches of 50 and 97.0-97.9 from
        # the sixth on (about 25 ms of the same load).  Untimed batches until 40 ms of launches have gone by (12
        # batches at most), then the timed one.
        spent = 0.0
        for _ in range(12):
            ms, _, _ = eng.time_kernel(which, args.kernel_reps)
            spent += ms * args.kernel_reps
            if spent >= 40.0:
                break
        return eng.time_kernel(which, args.kernel_reps)

    if args.kernel_pass:
        # every kernel family the timing aid knows, alone, back to back: the shape the rocprofv3 --pmc passes
        # of profiles/ are taken in (per family: 1 warm-up + --kernel-reps launches, in this order)
        shared_step(0)
        eng.sync()
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")     # counter calibration: 1 GiB read + 1 GiB written
        b = torch.empty_like(a)
        a.fill_(1.0)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        fams = ["qkv_gemm", "attention", "layernorm", "depth_conv3x3", "depth_fuse_upsample", "proj_gemm", "fc1_gemm", "fc2_gemm",
                "standalone_activation", "fc1_gemm_no_activation"]
        rows = {}
        for which, name in enumerate(fams):
            if which in (3, 4) and "depth" not in kinds:
                continue
            ms, fl, by = eng.time_kernel(which, args.kernel_reps)
            rows[name] = {"us": round(ms * 1e3, 2), "tflops": round(fl / ms / 1e9, 2), "gbps": round(by / ms / 1e6, 1),
                          "algorithmic_flops": fl, "algorithmic_bytes": by}
        print(json.dumps({"mode": "kernel-pass", "workload": spec.name, "reps": args.kernel_reps, "kernels": rows}))
        eng.close()
        return

    if args.roofline_only:
        shared_step(0)
        eng.sync()
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read + 1 GiB written
        b = torch.empty_like(a)
        a.fill_(1.0)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        ms, fl, by = settled_kernel_time(3 if "depth" in kinds else 0)
        print(json.dumps({"mode": "roofline-only", "kernel_us": round(ms * 1e3, 2), "tflops": round(fl / ms / 1e9, 2),
                          "algorithmic_bytes": by, "copy_bytes_each_way": 4 * a.numel()}))
        eng.close()
        return

    t_shared, t_shared_bracketed = timed(shared_step, args.steps, args.warmup)

    # the same step fed from raw camera frames (paper: 1920x1080 streams): uint8 -> resize -> normalise on the GPU
    # in front of the encoder, each frame on the engine stream its encoder pass will use
    cams = [torch.from_numpy(vi.make_camera_frame(1080, 1920, iseed + 100 + i)[None].repeat(spec.batch, axis=0)).cuda() for i in range(2)]
    # one image buffer per encoder lane: the transform of frame i runs on the stream of lane i % lanes, after that
    # lane's previous encoder pass (frame i - lanes), the only reader of the buffer it overwrites
    cam_imgs = [torch.empty_like(frames[0]) for _ in range(args.encoder_lanes)]

    def camera_step(i):
        img = cam_imgs[eng.stats()[0] % args.encoder_lanes]
        vpe.preprocess_u8(cams[i & 1], img, vi.CAMERA_MEAN, vi.CAMERA_STD, stream=eng.next_encode_stream())
        fh = eng.encode(img)
        for h in range(nh):
            eng.run_head(h, fh)

    t_cam, _ = timed(camera_step, args.steps, args.warmup)
    t_seq, _ = timed(sequential_step, max(args.steps // 3, 10), max(args.warmup // 3, 3))
    t_ind, _ = timed(independent_pipelined_step, max(args.steps // 3, 10), max(args.warmup // 3, 3))
    t_enc, _ = timed(encode_step, args.steps, args.warmup)
    fps = spec.batch / t_shared

    # unloaded latency of one frame as the host sees it: submit encode + heads on an idle GPU, wait for all
    lat = []
    for i in range(min(args.steps, 100)):
        t0 = time.perf_counter()
        shared_step(i)
        eng.sync()
        lat.append((time.perf_counter() - t0) * 1e3)
    lat.sort()
    latency = {"p10": round(lat[len(lat) // 10], 4), "median": round(lat[len(lat) // 2], 4), "p90": round(lat[(9 * len(lat)) // 10], 4)}
    bb_tflops = backbone_flops(spec) / t_enc / 1e12

    # roofline of the dominant kernel: the depth head's largest 3x3 convolution (implicit GEMM on MFMA,
    # 43 % of the frame's FLOP in one launch), timed with HIP events on the stream it is launched on
    roofline = None
    kern = {}
    shared_step(0)
    eng.sync()
    for which, name in ((0, "qkv_gemm"), (1, "attention"), (2, "layernorm"), (5, "proj_gemm"), (6, "fc1_gemm"), (7, "fc2_gemm"), (8, "standalone_activation"), (9, "fc1_gemm_no_activation")) + (((3, "depth_conv3x3"), (4, "depth_fuse_upsample")) if "depth" in kinds else ()):
        ms, fl, by = settled_kernel_time(which)
        kern[name] = {"us": round(ms * 1e3, 2), "tflops": round(fl / ms / 1e9, 2), "gbps": round(by / ms / 1e6, 1)}
        if name in ("layernorm", "depth_fuse_upsample", "standalone_activation"):            # bandwidth-bound kernels: fraction of the 8 TB/s HBM peak
            kern[name]["hbm_frac"] = round(by / ms / 1e6 / 8000.0, 4)
        if name == "depth_conv3x3" or (name == "qkv_gemm" and "depth" not in kinds):
            peak = MFMA_PEAK_TFLOPS[spec.dtype]
            ach = fl / (ms * 1e-3) / 1e12
            roofline = {"kernel": name, "bound": "mfma", "achieved": round(ach, 2), "peak": peak, "unit": "TFLOP/s",
                        "frac": round(ach / peak, 4),
                        "traffic": args.traffic_bytes if args.traffic_bytes is not None else (measured_traffic(name, spec.name) if not args.head_ch else None),
                        "us_per_launch": round(ms * 1e3, 2),
                        "algorithmic_bytes": by, "algorithmic_flops": fl}

    # the same step on an engine created with the library's defaults (one encoder lane, ring of two, as many head
    # streams as heads): what an application gets without choosing lanes, ring and hardware queues
    eng.close()
    eng, _, _ = make_engine(spec, wseed, kinds=kinds, ring_slots=2, flags=flags, encoder_lanes=1, weights=w)
    lanes_used, args.encoder_lanes = args.encoder_lanes, 1
    t_default, _ = timed(shared_step, max(args.steps // 3, 10), max(args.warmup // 3, 3))
    args.encoder_lanes = lanes_used

    cpu_baseline = None
    if not args.no_cpu_baseline:
        # the oracle as it stands, on this machine's host cores: one frame (batch element 0) of the same workload
        from oracle import model, ops
        t0 = time.perf_counter()
        feats = model.encode_image(spec, w, images_np[0])
        for k, hwd in zip(kinds, hw):
            {"seg": model.seg_head, "depth": model.depth_head, "det": model.det_head, "dpt": model.dpt_head}[k](spec, hwd, feats)
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": round(1.0 / dt, 5), "unit": "frames/s", "cores": ops.num_threads(), "kind": "oracle",
                        "sample": f"1 frame (batch element 0) of {spec.name}, encoder + {nh} head(s), {dt:.1f} s"}

    out = {
        "metric": "end-to-end frames/sec (backbone+3 heads), ViT-S/14 476x630; backbone TFLOP/s",
        "value": round(fps, 2), "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_shared * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": spec.name, "batch": spec.batch, "img": [spec.img_h, spec.img_w], "tokens": spec.tokens,
                   "heads": list(kinds), "ring_slots": args.ring_slots, "encoder_lanes": args.encoder_lanes, "head_streams": head_streams,
                   "hw_queues": args.hw_queues, "hip_graphs": not args.no_graphs, "timing": "steady state: (t(prime + steps) - t(prime)) / steps"},
        "backbone_tflops": round(bb_tflops, 2), "backbone_ms": round(t_enc * 1e3, 4),
        "backbone_mfma_frac": round(bb_tflops / MFMA_PEAK_TFLOPS[spec.dtype], 4),
        "from_1080p_uint8_fps": round(spec.batch / t_cam, 2),
        "library_defaults_fps": round(spec.batch / t_default, 2),
        "fps_incl_fill_and_drain": round(spec.batch / t_shared_bracketed, 2),
        # sequential baseline (each head recomputes its own backbone pass): on one stream, one frame at a time, and
        # with the same lanes / streams / queues as the shared path; the like-for-like ratios are latency against
        # latency and pipelined against pipelined
        "sequential_baseline_fps": round(spec.batch / t_seq, 2), "sequential_baseline_pipelined_fps": round(spec.batch / t_ind, 2),
        "shared_vs_sequential": round(t_ind / t_shared, 3),
        "shared_vs_sequential_latency": round(t_seq * 1e3 / latency["median"], 3),
        "shared_pipelined_vs_sequential_one_stream": round(t_seq / t_shared, 3),
        "frame_latency_ms": latency, "kernels": kern, "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))
    eng.close()


if __name__ == "__main__":
    main()
