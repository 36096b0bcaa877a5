#!/usr/bin/env python3
"""Benchmark of the per-frame tool-tracking hot path on one MI355X.

A step is one pass of all four stages (format conversion + resize, ResNet-18-style backbone +
ConvLSTM + head on fp16 MFMA, postprocess, overlay) over one batch of input: one 1920x1080
frame of every stream the workload serves.  Frames are synthetic and already resident in HBM
when the timed region starts.

Without workload flags the run covers the benchmark's configurations in one process and prints
ONE JSON line:
  * headline (`value`, `config`, `latency_ms`, `roofline`, `kernels`): twelve concurrent 1080p
    streams at 30 frames per second each, batched across streams through one pass of the network
    (the largest single-GPU configuration);
  * `configs`: short runs of the other configurations -- one stream; five unpartitioned
    applications at 60 frames per second; six applications unpartitioned, on six CU partitions
    with inference and overlay on separate CU sets, on six partitions with one queue each, and
    re-shaped into three applications of two streams on three partitions and two applications
    of three streams on two partitions -- each with frames/s
    and the latency determinism metrics (paper Section V-A); the six-stream arrangements carry
    their maximum and median against the unpartitioned run's and the Mann-Whitney z of the two
    latency samples (paper, appendix "Additional Evaluation");
  * `cpu_baseline`: the CPU oracle timed on the host's cores.
With workload flags (--streams, --batch, --partition, ...) it measures that one workload.
"""
from __future__ import annotations

import argparse
import copy
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0   # MI355X dense fp16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
FW, FH, NW, NH = 1920, 1080, 854, 480

WORKLOAD_FLAGS = ("--streams", "--batch", "--partition", "--partition-groups", "--tiny-groups",
                  "--hog", "--tiny-apps", "--group-nets", "--per-stream-submit", "--annotate",
                  "--fps", "--first-seed")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default: 100 batches of the headline workload, 240 frames "
                         "of a workload given by flags)")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--streams", type=int, default=1, help="concurrent applications")
    ap.add_argument("--batch", type=int, default=1,
                    help="streams per application, batched through the network together "
                         "(--streams counts applications; 12 with --fps 30 is the saturation case)")
    ap.add_argument("--fps", type=float, default=60.0, help="pacing of the latency run")
    ap.add_argument("--first-seed", type=int, default=None,
                    help="scene seed of the first stream (default: 1 for a single stream, else 2)")
    ap.add_argument("--partition", choices=["none", "equal", "equal-shared"], default="none",
                    help="equal: disjoint CU-masked partitions, inference and overlay on separate "
                         "CU sets and queues; equal-shared: one CU set and one queue per "
                         "application for all four stages")
    ap.add_argument("--partition-groups", type=int, default=0, metavar="G",
                    help="with --partition equal: CU groups (8 CUs, one per XCD) per application "
                         "instead of an equal share of the device; the last group serves the overlay")
    ap.add_argument("--tiny-groups", type=int, default=0, metavar="G",
                    help="with a partition and --tiny-apps: CU groups per small-network application; "
                         "the other applications share the rest equally")
    ap.add_argument("--hog", type=int, default=0, metavar="K",
                    help="K extra applications that submit frames back to back during the paced "
                         "latency run (saturating neighbours, not counted in the latency figures); "
                         "with --partition equal they get partitions of their own")
    ap.add_argument("--tiny-apps", type=int, default=0, metavar="K",
                    help="K applications of the small network (320x240 frames -> 128x128, 4 conv "
                         "layers) paced beside the others during the latency run: heterogeneous "
                         "applications sharing the GPU; their latencies are reported separately")
    ap.add_argument("--pin-cpus", action="store_true",
                    help="pin every application's submitting thread and completion thread to cores "
                         "of their own (cores 2i and 2i+1 of this process's CPU set)")
    ap.add_argument("--save-latencies", metavar="FILE",
                    help="write the trimmed per-frame latencies (ms) of the paced run as JSON")
    ap.add_argument("--compare-latencies", metavar="FILE",
                    help="Mann-Whitney U of this run's latencies against a file written by "
                         "--save-latencies (|z| > 1.96: the distributions differ)")
    ap.add_argument("--annotate", action="store_true",
                    help="overlay also draws argmax markers and tool labels (off in the headline "
                         "workload)")
    ap.add_argument("--group-nets", type=int, default=1, metavar="N",
                    help="every application runs N networks side by side on each frame and draws "
                         "their layers in one overlay launch (the paper's multi-network "
                         "application, Section III-B); needs --batch 1")
    ap.add_argument("--per-stream-submit", action="store_true",
                    help="with --batch B > 1: every stream of a batch submits its own frame from "
                         "its own thread (hs_mux); latency then counts from the stream's own "
                         "arrival and includes the wait for the rest of the batch")
    ap.add_argument("--paced-frames", type=int, default=60)
    ap.add_argument("--repeats", type=int, default=None,
                    help="repeat the paced latency run this many times (state reset in between) "
                         "and pool the trimmed latencies, as the paper pools its repeated runs "
                         "(default 3; 2 per configuration in the run over all configurations)")
    ap.add_argument("--distinct-frames", type=int, default=None,
                    help="distinct frames per stream, cycled (default 8; 4 and 2 in the run over "
                         "all configurations)")
    ap.add_argument("--queue-depth", type=int, default=4)
    ap.add_argument("--launch-mode", choices=["graph", "eager"], default="eager",
                    help="stages 1-3 kernel by kernel (the library's default: lowest latency), "
                         "or as one HIP graph per frame")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="first run the library's plain copy kernel 4 times over this many MiB "
                         "(reference dispatches for scaling rocprofv3 byte counters)")
    ap.add_argument("--headline-only", action="store_true",
                    help="default run without the configs array: the headline measurement alone, "
                         "unchanged (the command the kernel-trace profile of the headline uses)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-frames", type=int, default=16,
                    help="frames of the all-core CPU oracle sample (one more, untimed, first)")
    ap.add_argument("--cpu-frames-1thread", type=int, default=2,
                    help="frames of the single-thread CPU oracle sample")
    return ap.parse_args()


def equal_partitions(n_cus: int, n_streams: int, overlay_groups: int = 1, spare_groups: int = 2,
                     n_xcd: int = 8, groups_per_app: int = 0):
    """n_streams disjoint CU sets of equal size, built from groups of n_xcd consecutive CUs
    (CU i sits on XCD i mod n_xcd and a mask needs a CU on every XCD).  Inside each set the
    last overlay_groups groups serve the overlay stream, the rest the inference stream;
    spare_groups groups stay unclaimed (the paper's appendix recommends leaving headroom)."""
    groups = n_cus // n_xcd - spare_groups
    per = groups_per_app if groups_per_app else groups // n_streams
    if per < 2 or per * n_streams > n_cus // n_xcd:
        raise SystemExit(f"{n_streams} partitions of {per} CU groups do not fit {n_cus} CUs")
    parts = []
    for i in range(n_streams):
        cus = list(range(i * per * n_xcd, (i + 1) * per * n_xcd))
        k = overlay_groups * n_xcd
        parts.append((cus[:-k], cus[-k:]))
    return parts


class Env:
    """What every measured workload shares: the library context, the weight blob and a cache
    of generated scenes (so that arrangements of the same streams reuse their frames)."""

    def __init__(self):
        import numpy as np
        import torch
        import paper_2402_04466_amd as hs
        import synth_inputs as si
        self.np, self.torch, self.hs, self.si = np, torch, hs, si
        self.ctx = hs.hs_init(0)
        self.n_cus = hs.hs_device_cus(self.ctx)
        self.blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
        self._scenes = {}

    def scene(self, seed: int, n: int):
        key = (seed, n)
        if key not in self._scenes:
            self._scenes[key] = list(self.si.tool_scene_frames(n, FH, FW, seed))
        return self._scenes[key]


def measure(args, env: Env, want_roofline: bool = True, note=lambda s: None) -> dict:
    """One workload: throughput back to back, latency determinism at the paced rate, per-kernel
    timing of its first application.  Creates and destroys its applications."""
    hs, np, torch, si, ctx, n_cus = env.hs, env.np, env.torch, env.si, env.ctx, env.n_cus
    from paper_2402_04466_amd.harness import AppStream, GroupStream, run_paced
    from paper_2402_04466_amd.harness import run_back_to_back as harness_back_to_back
    blob = env.blob
    grouped = args.group_nets > 1
    if grouped and args.batch != 1:
        raise SystemExit("--group-nets needs --batch 1")
    first_seed = args.first_seed if args.first_seed is not None else \
        (1 if args.streams * args.batch == 1 else 2)

    def apps_of(s):
        """The library applications behind one benchmark stream."""
        return [m.app for m in s.members] if isinstance(s, GroupStream) else [s.app]

    streams, frames = [], []
    for i in range(args.streams):
        members = []
        for j in range(args.group_nets):
            # members of a group differ in weights (seed) and colours, not in architecture
            members.append(AppStream(
                ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=FW, frame_h=FH, net_w=NW, net_h=NH,
                blob=blob if j == 0 else si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1 + j),
                palette=np.roll(si.DEFAULT_PALETTE, j, axis=0).copy(),
                queue_depth=args.queue_depth, batch=args.batch,
                glyphs=si.DEFAULT_GLYPHS if args.annotate else None))
            hs.hs_set_launch_mode(members[-1].app, hs.HS_LAUNCH_GRAPH
                                  if args.launch_mode == "graph" else hs.HS_LAUNCH_EAGER)
        s = GroupStream(ctx, members) if grouped else members[0]
        streams.append(s)
        per_stream = []
        for j in range(args.batch):
            seed = first_seed + i * args.batch + j
            per_stream.append([s.upload_frame(f) for f in env.scene(seed, args.distinct_frames)])
        # frames[i][k] = what is submitted as frame k of application i (one tensor per stream)
        frames.append([[per_stream[j][k] for j in range(args.batch)]
                       for k in range(args.distinct_frames)])
    hogs, hog_frames, hog_outs = [], [], []
    for i in range(args.hog):
        s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=FW, frame_h=FH, net_w=NW,
                      net_h=NH, blob=blob, palette=si.DEFAULT_PALETTE,
                      queue_depth=args.queue_depth, batch=1)
        hogs.append(s)
        hog_frames.append([s.upload_frame(f) for f in env.scene(100 + i, 2)])
        hog_outs.append([s.new_output() for _ in range(args.queue_depth)])
    tiny, tiny_frames, tiny_outs = [], [], []
    if args.tiny_apps:
        tiny_blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
        for i in range(args.tiny_apps):
            s = AppStream(ctx, net=hs.HS_NET_TINY4, frame_w=320, frame_h=240, net_w=128, net_h=128,
                          blob=tiny_blob, palette=si.DEFAULT_PALETTE, queue_depth=args.queue_depth,
                          net_fp32_input=True)
            tiny.append(s)
            tiny_frames.append([[s.upload_frame(f)] for f in si.uniform_frames(8, 240, 320, 50 + i)])
            tiny_outs.append([[s.new_output()] for _ in range(args.queue_depth)])
    part_cus = {}     # library application -> (CUs of its inference mask, of its overlay mask)
    if args.partition != "none" and args.tiny_groups and tiny:
        # unequal slices: G groups per small application, the rest split among the others
        n_big = args.streams + args.hog
        total_groups = n_cus // 8
        big_groups = (total_groups - args.tiny_groups * len(tiny)) // max(n_big, 1)
        if big_groups < 2 or args.tiny_groups < 2:
            raise SystemExit("partition sizes do not fit (every application needs >= 2 CU groups)")
        if grouped:
            raise SystemExit("--tiny-groups is not combined with --group-nets")
        at = 0
        for s in streams + hogs + tiny:
            g = args.tiny_groups if s in tiny else big_groups
            cus = list(range(at * 8, (at + g) * 8))
            at += g
            ci, co = (cus, cus) if args.partition == "equal-shared" else (cus[:-8], cus[-8:])
            hs.hs_set_partition(s.app, hs.cu_mask_words(ci), hs.cu_mask_words(co))
            part_cus[s.app] = (len(ci), len(co))
    elif args.partition != "none":
        # one partition per library application (every network of a group gets its own)
        units = [a for s in streams + tiny + hogs for a in apps_of(s)]
        for a, (ci, co) in zip(units, equal_partitions(n_cus, len(units),
                                                       groups_per_app=args.partition_groups)):
            if args.partition == "equal-shared":
                ci = co = ci + co
            hs.hs_set_partition(a, hs.cu_mask_words(ci), hs.cu_mask_words(co))
            part_cus[a] = (len(ci), len(co))
    outs = [[[s.new_output() for _ in range(args.batch)] for _ in range(args.queue_depth)]
            for s in streams]
    torch.cuda.synchronize()

    def run_back_to_back(n_frames: int):
        """Every stream submits n_frames as fast as its queue allows (the library's native
        driver, one submitting thread per application).  Returns elapsed s: the driver's own
        clock from starting the submitting threads to collecting the last result, bracketed by
        device synchronisation on both sides (the interpreter's pauses -- a garbage collection
        can take 40 ms -- stay out of the timed region)."""
        torch.cuda.synchronize()
        _, elapsed = harness_back_to_back(streams, frames, outs, n_frames)
        torch.cuda.synchronize()
        return elapsed

    # ---- throughput: W warm-up steps, then exactly K timed steps per application -------------
    if args.warmup > 0:
        run_back_to_back(args.warmup)
    elapsed = run_back_to_back(args.steps)
    total_frames = args.steps * args.streams * args.batch
    fps = total_frames / elapsed
    note("throughput done")

    # ---- latency determinism at a fixed frame rate (paper Section V-A metrics) -------------
    for s in streams:
        for a in apps_of(s):
            hs.hs_reset_state(a)
    paced = [(f * ((args.paced_frames + len(f) - 1) // len(f)))[:args.paced_frames]
             for f in frames]
    hog_stop = threading.Event()
    hog_count = [0] * len(hogs)

    def hog_worker(i):
        s, k, inflight = hogs[i], 0, 0
        while not hog_stop.is_set():
            if s.submit(hog_frames[i][k % 2], hog_outs[i][k % args.queue_depth], k) == hs.HS_OK:
                k += 1
                inflight += 1
            else:
                s.wait()
                inflight -= 1
                hog_count[i] += 1
        for _ in range(inflight):
            s.wait()

    hog_threads = [threading.Thread(target=hog_worker, args=(i,)) for i in range(len(hogs))]
    for t in hog_threads:
        t.start()
    t_hog = time.perf_counter()
    pins = None
    if args.pin_cpus:
        cores = sorted(os.sched_getaffinity(0))
        pins = [cores[(2 * i) % len(cores)] for i in range(len(streams) + len(tiny))]
        for i, s in enumerate(streams + tiny):
            for a in apps_of(s):
                hs.hs_set_cpu_affinity(a, cores[(2 * i + 1) % len(cores)])
    tiny_paced = [(f * ((args.paced_frames + len(f) - 1) // len(f)))[:args.paced_frames]
                  for f in tiny_frames]
    muxes = None
    if args.per_stream_submit and args.batch > 1 and not grouped:
        muxes = [hs.hs_create_mux(s.app, args.batch) for s in streams]
    lat_ms, tl, dropped, results, kept, lateness_us = [], [], [], [], [], []
    for rep in range(max(1, args.repeats)):
        if rep:
            for s in streams + tiny:
                for a in apps_of(s):
                    hs.hs_reset_state(a)
        res_all, drop, late = run_paced(streams + tiny, paced + tiny_paced, args.fps,
                                        outs + tiny_outs, pin_cpus=pins,
                                        n_frames=args.paced_frames, with_lateness=True,
                                        muxes=muxes + [None] * len(tiny) if muxes else None)
        note(f"paced run {rep + 1} of {max(1, args.repeats)} done")
        lateness_us.extend(v / 1e3 for per in late for v in per)
        dropped.extend(drop)
        tiny_results, results = res_all[len(streams):], res_all[:len(streams)]
        for rs in tiny_results:
            per = [(r[0].t_overlay_done_ns - r[0].t_submit_ns) / 1e6 for r in rs]
            t = min(10, len(per) // 6)
            tl.extend(per[t:len(per) - t])
        for rs in results:
            t = min(10, len(rs) // 6)
            kept.extend((rep, k, r[0]) for k, r in list(enumerate(rs))[t:len(rs) - t])
            for j in range(args.batch):
                per = [(r[j].t_overlay_done_ns - r[j].t_submit_ns) / 1e6 for r in rs]
                lat_ms.extend(per[t:len(per) - t])   # trim each stream's warm-up / cool-down
    tiny_m = None
    if tiny:
        tm = hs.hs_latency_metrics_compute(tl, trim=False)
        tiny_m = {k: (int(v) if k == "n" else round(v, 4)) for k, v in tm.items()}
    for m in muxes or []:
        hs.hs_destroy_mux(m)
    hog_stop.set()
    for t in hog_threads:
        t.join()
    t_hog = time.perf_counter() - t_hog
    m = hs.hs_latency_metrics_compute(lat_ms, trim=False)
    mwu = None
    if args.compare_latencies:
        with open(args.compare_latencies) as fh:
            other = json.load(fh)
        mwu = hs.hs_mann_whitney_u(lat_ms, other["latency_ms"])
        mwu["against"] = other.get("label", args.compare_latencies)
    if args.save_latencies:
        with open(args.save_latencies, "w") as fh:
            json.dump({"label": " ".join(sys.argv[1:]), "latency_ms": lat_ms}, fh)
    per_stream_p50 = []
    for rs in results:
        for j in range(args.batch):
            per = [(r[j].t_overlay_done_ns - r[j].t_submit_ns) / 1e6 for r in rs]
            per_stream_p50.append(round(float(np.median(per)), 4))
    stage_ms = {}
    for name, a, b in (("pre", "t_submit_ns", "t_pre_done_ns"),
                       ("infer", "t_pre_done_ns", "t_infer_done_ns"),
                       ("post", "t_infer_done_ns", "t_post_done_ns"),
                       ("overlay", "t_post_done_ns", "t_overlay_done_ns")):
        v = [(getattr(r[0], b) - getattr(r[0], a)) / 1e6 for rs in results for r in rs]
        stage_ms[name] = round(float(np.median(v)), 4)
    # where the slowest kept frame spent its time (a late completion stamp, i.e.
    # host scheduling, shows up in "pre": the stage stamps are derived backwards from it)
    w_rep, w_k, worst = max(kept, key=lambda e: e[2].t_overlay_done_ns - e[2].t_submit_ns)
    worst_ms = {"pre": (worst.t_pre_done_ns - worst.t_submit_ns) / 1e6,
                "infer": (worst.t_infer_done_ns - worst.t_pre_done_ns) / 1e6,
                "post": (worst.t_post_done_ns - worst.t_infer_done_ns) / 1e6,
                "overlay": (worst.t_overlay_done_ns - worst.t_post_done_ns) / 1e6,
                "enqueue": (worst.t_enqueued_ns - worst.t_submit_ns) / 1e6}
    worst_ms = {k: round(v, 4) for k, v in worst_ms.items()}
    worst_ms["repeat"], worst_ms["frame"] = w_rep, w_k

    # ---- roofline of the dominant kernel: HIP events attached to every launch ----------------
    s0 = streams[0]
    app0 = apps_of(s0)[0]     # a group: its first network (and the shared overlay launch)
    roof, kernels, kt = None, {}, []
    if want_roofline:
        # the paced run leaves the GPU idle most of the time and its clocks low: a short
        # back-to-back burst brings them back up before the per-launch timing (untimed)
        harness_back_to_back(streams[:1], frames[:1], outs[:1], 60)
        hs.hs_set_kernel_timing(app0, True)
        n_prof = 40
        for k in range(n_prof):
            assert s0.submit_batch(frames[0][k % len(frames[0])], outs[0][k % len(outs[0])],
                                   k) == hs.HS_OK
            s0.wait_batch()
        kt = hs.hs_get_kernel_times(app0)
        hs.hs_set_kernel_timing(app0, False)
        dom = max(kt, key=lambda e: e["total_ms"])
        if dom["flops"] > 0:
            ach = dom["flops"] / (dom["total_ms"] * 1e-3) / 1e12
            roof = {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_FP16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(ach / PEAK_FP16_TFLOPS, 4), "traffic": None}
        else:
            ach = dom["bytes"] / (dom["total_ms"] * 1e-3) / 1e9
            roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None}
        # HBM bytes per launch: not measured in this run.  They come from committed rocprofv3
        # counter runs and are given only while the kernel sources still hash to what those
        # runs recorded.
        roof["traffic_source"] = None
        try:
            from paper_2402_04466_amd.pmc_traffic import kernel_source_hash
            tag = "config2_1stream" if args.streams * args.batch == 1 else f"batch{args.batch}"
            rel = os.path.join("profiles", f"conv_traffic_{tag}.json")
            with open(os.path.join(ROOT, rel)) as fh:
                tr = json.load(fh)
            if tr["kernel_source_sha256"] == kernel_source_hash() and dom["name"] == "conv_mfma":
                roof["traffic"] = round(tr["conv_hbm_bytes_per_launch"]["total"])
                roof["traffic_source"] = rel + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an " \
                                               "earlier run of this kernel source, not this run)"
        except (OSError, KeyError, ValueError):
            pass
        roof["kernel"] = dom["name"]
        roof["avg_launch_us"] = round(dom["total_ms"] * 1e3 / dom["launches"], 2)
        roof["launches_per_step"] = dom["launches"] // n_prof
        roof["frames_per_launch"] = args.batch
        for e in kt:
            d = {"us_per_step": round(e["total_ms"] * 1e3 / n_prof, 2),
                 "launches_per_step": e["launches"] // n_prof}
            if e["flops"] > 0:
                d["TFLOP/s"] = round(e["flops"] / (e["total_ms"] * 1e-3) / 1e12, 2)
            if e["bytes"] > 0:
                d["GB/s"] = round(e["bytes"] / (e["total_ms"] * 1e-3) / 1e9, 1)
            kernels[e["name"]] = d

    # what the first application's share of the device can pull and compute: a plain copy of the
    # overlay's shape under the same CU mask, and the fp16 MFMA peak of its CUs
    part = None
    if args.partition != "none":
        per_app = args.batch * FH * s0.frame_pitch
        src = torch.full((per_app,), 3, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        sec = hs.hs_partition_copy(app0, dst.data_ptr(), src.data_ptr(), per_app, 20)
        copy_gbs = 2.0 * per_app / sec / 1e9
        cus = part_cus.get(app0)
        part = {"application": 0, "cus_inference": cus[0], "cus_overlay": cus[1],
                "copy_GB/s": round(copy_gbs, 1)}
        ov = next((e for e in kt if e["name"] == "overlay"), None)
        if ov and ov["total_ms"] > 0:
            ov_gbs = ov["bytes"] / (ov["total_ms"] * 1e-3) / 1e9
            part["overlay_GB/s"] = round(ov_gbs, 1)
            part["overlay_vs_copy"] = round(ov_gbs / copy_gbs, 3)
        cv = next((e for e in kt if e["name"] == "conv_mfma"), None)
        if cv and cv["total_ms"] > 0:
            peak = cus[0] * PEAK_FP16_TFLOPS / 256.0
            ach = cv["flops"] / (cv["total_ms"] * 1e-3) / 1e12
            part["conv_TFLOP/s"] = round(ach, 2)
            part["conv_peak_of_its_cus_TFLOP/s"] = round(peak, 1)
            part["conv_frac_of_its_cus"] = round(ach / peak, 4)
        del src, dst
    hog_rate = round(sum(hog_count) / t_hog, 1) if hogs else None
    for s in streams + tiny + hogs:
        s.close()

    n_streams = args.streams * args.batch
    return {
        "value": round(fps, 2), "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * elapsed / args.steps, 4),
        "config": {"workload": f"{n_streams} stream(s) x 1920x1080 RGB uint8 -> 854x480 fp16, "
                               "ResNet-18-style + ConvLSTM(256) + 8-ch head, sigmoid/threshold/"
                               "argmax, alpha-blend overlay on the 1080p frame"
                               + (f"; {args.batch} streams batched through one pass of the network "
                                  "per application" if args.batch > 1 else "")
                               + (f"; {args.group_nets} such networks per stream, one overlay "
                                  "launch for their layers" if grouped else ""),
                   "streams": n_streams, "applications": args.streams, "batch": args.batch,
                   "group_nets": args.group_nets, "paced_fps": args.fps,
                   "first_seed": first_seed, "per_stream_submit": bool(muxes),
                   "partition": args.partition, "partition_groups": args.partition_groups,
                   "queue_depth": args.queue_depth, "launch_mode": args.launch_mode,
                   "hog_apps": args.hog, "tiny_apps": args.tiny_apps,
                   "tiny_groups": args.tiny_groups, "annotate": bool(args.annotate),
                   "device_cus": n_cus},
        "latency_ms": {"paced_fps": args.fps, "frames": int(m["n"]), "repeats": max(1, args.repeats),
                       "p50": round(m["p50"], 4), "p99": round(m["p99"], 4),
                       "p999": round(float(np.percentile(lat_ms, 99.9)), 4),
                       "above_2x_p50": int(np.sum(np.asarray(lat_ms) > 2.0 * m["p50"])),
                       "max": round(m["max"], 4), "mean": round(m["mean"], 4),
                       "std": round(m["std"], 4), "tail": round(m["tail"], 4),
                       "flatness": round(m["flatness"], 4), "dropped": int(sum(dropped)),
                       "submit_lateness_us": {"p50": round(float(np.median(lateness_us)), 1),
                                              "max": round(float(np.max(lateness_us)), 1)},
                       "stage_median_ms": stage_ms, "slowest_frame_stage_ms": worst_ms,
                       "per_stream_p50": per_stream_p50,
                       "mann_whitney": mwu, "pinned_cpus": bool(args.pin_cpus),
                       "tiny_apps": tiny_m,
                       "hog_frames_per_s": hog_rate},
        "roofline": roof,
        "partition_share": part,
        "kernels": kernels,
        "_lat_ms": lat_ms,
    }


def cpu_baseline(args, env: Env) -> dict:
    """The CPU oracle as it stands on the host's cores: all four stages of one 1080p
    stream, with every core the BLAS library takes, and on a single thread."""
    import oracle
    si = env.si
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    app = oracle.OracleApp("resnet18_convlstm", env.blob, NW, NH, True, si.DEFAULT_PALETTE)
    fr = list(si.tool_scene_frames(args.cpu_frames + 1, FH, FW, 1))
    app.process(fr[0])                       # first call pays one-time page-in costs
    t0 = time.perf_counter()
    for f in fr[1:]:
        app.process(f)
    dt = time.perf_counter() - t0
    cpu = {"value": round((len(fr) - 1) / dt, 4), "unit": "frames/s", "cores": int(cores),
           "kind": "oracle",
           "sample": f"{len(fr) - 1} frames of one 1080p stream of the same workload, all four "
                     "stages, NumPy float64; `cores` = BLAS threads (the integer stages run on "
                     "one)"}
    if threadpool_limits is not None and args.cpu_frames_1thread > 0:
        with threadpool_limits(limits=1):
            n1 = min(args.cpu_frames_1thread, len(fr) - 1)
            t0 = time.perf_counter()
            for f in fr[1:1 + n1]:
                app.process(f)
            dt1 = time.perf_counter() - t0
        cpu["single_thread"] = {"value": round(n1 / dt1, 4), "unit": "frames/s", "cores": 1,
                                "sample": f"{n1} frames of the same stream, BLAS limited to one "
                                          "thread"}
        cpu["one_stream_per_core_estimate"] = {
            "value": round(n1 / dt1 * (os.cpu_count() or 1), 3), "unit": "frames/s",
            "cores": os.cpu_count() or 1,
            "sample": "single-thread rate x host cores (streams are independent); not run"}
    return cpu


def summary(name: str, res: dict) -> dict:
    """The short form of a measured workload for the `configs` array."""
    lat = res["latency_ms"]
    out = {"name": name, "workload": res["config"]["workload"],
           "applications": res["config"]["applications"], "batch": res["config"]["batch"],
           "partition": res["config"]["partition"],
           "partition_groups": res["config"]["partition_groups"],
           "first_seed": res["config"]["first_seed"],
           "frames_per_s": res["value"], "steps": res["steps"], "ms_per_step": res["ms_per_step"],
           "latency_ms": {k: lat[k] for k in ("paced_fps", "frames", "repeats", "p50", "p99", "max",
                                              "mean", "std", "tail", "flatness", "dropped",
                                              "above_2x_p50")}}
    if res["partition_share"]:
        out["partition_share"] = res["partition_share"]
    if res["kernels"]:
        out["kernels"] = res["kernels"]
        out["roofline"] = res["roofline"]
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this library has no multi-GPU path (streams would "
              "shard one application per GPU with no communication); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    custom = any(a.split("=")[0] in WORKLOAD_FLAGS for a in sys.argv[1:])
    env = Env()
    hs, torch = env.hs, env.torch

    def note(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    if args.calibrate_copy:
        nbytes = args.calibrate_copy << 20
        a = torch.full((nbytes,), 7, dtype=torch.uint8, device="cuda:0")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(4):
            hs.hs_device_copy(env.ctx, b.data_ptr(), a.data_ptr(), nbytes)
        del a, b

    configs = None
    if custom:
        if args.steps is None:
            args.steps = 240
        if args.repeats is None:
            args.repeats = 3
        if args.distinct_frames is None:
            args.distinct_frames = 8
        head = measure(args, env, note=note)
    else:
        def variant(**kw):
            v = copy.copy(args)
            v.repeats = args.repeats if args.repeats is not None else 2
            v.distinct_frames = args.distinct_frames if args.distinct_frames is not None else 2
            for k, val in kw.items():
                setattr(v, k, val)
            return v

        # headline: configuration 5, twelve streams batched, 30 frames per second each
        h = variant(streams=1, batch=12, fps=30.0, first_seed=13,
                    steps=args.steps if args.steps is not None else 100,
                    distinct_frames=args.distinct_frames if args.distinct_frames is not None else 4)
        note("configuration 5: 12 streams batched, 30 fps")
        head = measure(h, env, note=note)
        torch.cuda.empty_cache()
        # the other configurations, short: 120 frames per application back to back, then the
        # paced run.  Arrangements of configuration 4 share seeds 7-12.
        plan = [
            ("config 2: 1 stream, 60 fps", dict(streams=1, batch=1, first_seed=1, steps=240)),
            ("config 3: 5 applications, 60 fps each, unpartitioned",
             dict(streams=5, batch=1, first_seed=2, steps=120)),
            ("config 4: 6 applications, 60 fps each, unpartitioned (the reference run)",
             dict(streams=6, batch=1, first_seed=7, steps=120)),
            ("config 4 as stated: 6 applications on 6 equal CU partitions, inference (32 CUs) and "
             "overlay (8 CUs) on separate CU sets and queues",
             dict(streams=6, batch=1, first_seed=7, steps=120, partition="equal")),
            ("config 4, one queue per partition: 6 applications on 6 equal CU partitions of 40 CUs",
             dict(streams=6, batch=1, first_seed=7, steps=120, partition="equal-shared")),
            ("config 4 re-shaped: 3 applications x 2 streams batched, on 3 CU partitions of 80 CUs "
             "(at most four hardware queues in use)",
             dict(streams=3, batch=2, first_seed=7, steps=120, partition="equal-shared")),
            ("config 4 re-shaped: 2 applications x 3 streams batched, on 2 CU partitions of 120 CUs",
             dict(streams=2, batch=3, first_seed=7, steps=120, partition="equal-shared")),
        ]
        configs, ref = ([], None) if not args.headline_only else (None, None)
        for name, kw in (plan if not args.headline_only else []):
            note(name)
            res = measure(variant(**kw), env, want_roofline=kw.get("streams") == 1, note=note)
            torch.cuda.empty_cache()
            entry = summary(name, res)
            if name.startswith("config 4"):
                if ref is None:
                    ref = res
                else:
                    z = hs.hs_mann_whitney_u(res["_lat_ms"], ref["_lat_ms"])
                    rl, l = ref["latency_ms"], res["latency_ms"]
                    entry["vs_unpartitioned"] = {
                        "max_ratio": round(l["max"] / rl["max"], 3),
                        "p50_ratio": round(l["p50"] / rl["p50"], 3),
                        "std_ratio": round(l["std"] / max(rl["std"], 1e-9), 3),
                        "flatness_ratio": round(l["flatness"] / max(rl["flatness"], 1e-9), 3),
                        "max_below_unpartitioned": bool(l["max"] < rl["max"]),
                        "mann_whitney_z": round(z["z"], 2), "significant": bool(z["significant"])}
            configs.append(entry)
    hs.hs_shutdown(env.ctx)

    cpu = None
    if not args.no_cpu_baseline:
        note("CPU oracle")
        cpu = cpu_baseline(args, env)

    line = {
        "metric": "aggregate frames/s + p50/max per-frame latency at N concurrent streams, 1 GPU",
        "value": head["value"], "unit": "frames/s", "n_gpus": 1, "steps": head["steps"],
        "warmup": head["warmup"], "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": head["config"],
        "latency_ms": head["latency_ms"],
        "roofline": head["roofline"],
        "partition_share": head["partition_share"],
        "kernels": head["kernels"],
        "cpu_baseline": cpu,
    }
    if configs is not None:
        line["configs"] = configs
    print(json.dumps(line))


if __name__ == "__main__":
    main()
