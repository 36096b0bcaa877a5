"""GPU parity tests: every stage of libhs (called through the C ABI via the binding)
against the CPU oracle on the same seeded inputs.  Integer stages bit-exact; network
outputs within 2e-2 of the fp32 oracle (max-norm relative) and within 1.2e-2 of the oracle's
fp16-storage emulation (tests/gpu_common.py holds the bounds and what each is tied to)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
import oracle
from gpu_common import (check_frame, make_oracles, rel_err, rms_rel, TOL_CELL, TOL_NET, TOL_STATE_RMS,
                        TOL_STATE_MAX)

pytestmark = pytest.mark.gpu
PAL = si.DEFAULT_PALETTE


@pytest.fixture(scope="module")
def ctx(hs):
    c = hs.hs_init(0)
    yield c
    hs.hs_shutdown(c)


def _run_stream(hs, ctx, *, net, net_name, frames, net_w, net_h, blob, fp32_input, depth=2,
                threshold=0.5, alpha=0.5, check_state=False, tag="", glyphs=None,
                marker=(12, 1, 2), emulate=True, storage_gap=None):
    """emulate: also run the oracle's fp16-storage mode beside the fp32 one.
    storage_gap: per frame, the max-norm distance of the oracle's own fp16-storage mode from its
    fp32 mode on the logits (a stored, oracle-only measurement).  Where its running maximum is
    beyond half the nominal 2e-2, no half-precision-storage implementation can be expected
    inside 2e-2 of the fp32 oracle in the max norm; the bound there is twice that running
    maximum, the rms bound stays 2e-2, and the recurrent state is held to its rms bound only."""
    from paper_2402_04466_amd.harness import AppStream
    fh, fw, _ = frames[0].shape
    s = AppStream(ctx, net=net, frame_w=fw, frame_h=fh, net_w=net_w, net_h=net_h, blob=blob,
                  palette=PAL, queue_depth=depth, net_fp32_input=fp32_input, threshold=threshold,
                  alpha=alpha, glyphs=glyphs, marker_arm=marker[0], marker_half=marker[1],
                  glyph_scale=marker[2])
    o32, o16 = make_oracles(net_name, blob, net_w, net_h, not fp32_input, PAL,
                            threshold=threshold, alpha=alpha)
    errs = []
    w16 = None
    if check_state:
        ws = oracle.split_blob(blob, oracle.ResNet18ConvLSTMNet.shapes())
        w16 = [w.astype(np.float16).astype(np.float32) for w in ws[-2:]]   # lstm, head
        h_prev = c_prev = None
    try:
        for i, f in enumerate(frames):
            print(f"[{tag}] frame {i} {fw}x{fh} -> {net_w}x{net_h}", flush=True)
            d_in, d_out = s.upload_frame(f), s.new_output()
            assert s.submit(d_in, d_out, i) == hs.HS_OK
            r = s.wait()
            assert r.frame_id == i
            assert r.t_submit_ns <= r.t_pre_done_ns <= r.t_infer_done_ns <= r.t_post_done_ns \
                <= r.t_overlay_done_ns <= r.t_observed_ns
            g = s.fetch(r, d_out)
            a, b = o32.process(f), (o16.process(f) if emulate else None)
            tol_net = TOL_NET
            if storage_gap is not None:
                envelope = float(np.max(storage_gap[:i + 1]))
                if envelope > 0.5 * TOL_NET:
                    tol_net = max(TOL_NET, 2.0 * envelope)
            errs.append(check_frame(g, f, a, b, threshold=threshold, alpha=alpha, palette=PAL,
                                    fp32_input=fp32_input, tag=f"{tag}/frame{i}", glyphs=glyphs,
                                    marker=marker, tol_net=tol_net))
            if check_state:
                gh, gc = s.state(r)
                gx = s.features(r)
                if h_prev is None:
                    h_prev, c_prev = np.zeros_like(gh), np.zeros_like(gc)
                # the recurrent cell and the head in isolation: the oracle's step on the GPU's
                # own fp16 inputs (features, previous state) and fp16-rounded weights
                oh, oc = oracle.convlstm_step(gx, h_prev, c_prev, w16[0])
                ol = oracle.conv2d(gh, w16[1], 1, 0)
                ech, ecc, ehd = rel_err(gh, oh), rel_err(gc, oc), rel_err(g["logits"], ol)
                print(f"[{tag}] cell in isolation: h {ech:.2e} c {ecc:.2e} head {ehd:.2e}",
                      flush=True)
                assert max(ech, ecc, ehd) <= TOL_CELL, f"{tag}: cell h {ech:.3e} c {ecc:.3e} head {ehd:.3e}"
                h_prev, c_prev = gh, gc
                # end to end against the fp32 oracle
                stats = [rel_err(gh, a["h"]), rel_err(gc, a["c"]), rms_rel(gh, a["h"]),
                         rms_rel(gc, a["c"])]
                print(f"[{tag}] state vs fp32 oracle: max-norm h {stats[0]:.2e} c {stats[1]:.2e}; "
                      f"rms h {stats[2]:.2e} c {stats[3]:.2e}", flush=True)
                # the max-norm bound is tied to a measurement over the first four frames of a
                # stream; the long run (whose first frames another test checks with it) holds
                # the state to the rms bound and to the cell-in-isolation check above
                tol_max = TOL_STATE_MAX[f"{net_w}x{net_h}"] if (storage_gap is None and i < 4) \
                    else np.inf
                assert max(stats[0], stats[1]) <= tol_max and \
                    max(stats[2], stats[3]) <= TOL_STATE_RMS, \
                    f"{tag}: recurrent state drift {stats}"
    finally:
        s.close()
    print(f"[{tag}] logits max-norm error vs fp32 oracle per frame: "
          + " ".join(f"{e:.2e}" for e in errs), flush=True)
    return errs


def test_config1_tiny_net_all_frames(hs, ctx):
    """8 frames 320x240 uniform random, 128x128 fp32 normalise, 4-layer net, 32x32x8 map."""
    frames = list(si.uniform_frames(8, 240, 320, 0))
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    _run_stream(hs, ctx, net=hs.HS_NET_TINY4, net_name="tiny4", frames=frames, net_w=128,
                net_h=128, blob=blob, fp32_input=True, tag="config1")


def test_resnet_convlstm_reduced_size_with_state(hs, ctx):
    """640x360 -> 288x160: several 64-pixel tiles per layer with ragged tails (M = 80*144,
    40*72, 20*36, 10*18, 5*9 = 45) and the ConvLSTM state carried over 4 frames."""
    frames = list(si.tool_scene_frames(4, 360, 640, 31))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    _run_stream(hs, ctx, net=hs.HS_NET_RESNET18_CONVLSTM, net_name="resnet18_convlstm",
                frames=frames, net_w=288, net_h=160, blob=blob, fp32_input=False,
                check_state=True, tag="resnet-small")


def test_resnet_convlstm_odd_map_sizes(hs, ctx):
    """324x180 -> 162x90: every map of the network has an odd side (45 x 81 convolution outputs
    under the pool, then 23 x 41, 12 x 21, 6 x 11 and 3 x 6 pixels), so the pooling window that
    hangs over the bottom and right edge, the stride-2 tiles' last row and column and the
    ragged 8 x 8 / 8 x 16 tiles are all met; two frames, every stage."""
    frames = list(si.tool_scene_frames(2, 180, 324, 33))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 2)
    _run_stream(hs, ctx, net=hs.HS_NET_RESNET18_CONVLSTM, net_name="resnet18_convlstm",
                frames=frames, net_w=162, net_h=90, blob=blob, fp32_input=False, tag="resnet-odd")


def test_config2_full_size_three_frames(hs, ctx):
    """1920x1080 -> 854x480, full network, 3 frames of the seed-1 scene with state."""
    frames = list(si.tool_scene_frames(3, 1080, 1920, 1))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    _run_stream(hs, ctx, net=hs.HS_NET_RESNET18_CONVLSTM, net_name="resnet18_convlstm",
                frames=frames, net_w=854, net_h=480, blob=blob, fp32_input=False,
                check_state=True, tag="config2")


@pytest.mark.timeout(600)
def test_config2_all_60_frames_with_carried_state(hs, ctx):
    """Configuration 2 at its stated length: 60 frames 1920x1080 of the seed-1 scene through the
    full network with the ConvLSTM state carried 0 -> 59, the fp32 oracle beside every frame.
    Every frame: stage 1 bit-exact; stages 3 and 4 bit-exact on the GPU's own logits / mask; the
    recurrent cell and the head, alone, on the GPU's own inputs within 2e-3 of the oracle's
    step -- so every one of the 60 state updates is checked by itself; logits against the fp32
    oracle within 2e-2 rms, and within 2e-2 in the max norm for as long as the oracle's own
    fp16-storage mode stays within 1e-2 of its fp32 mode (tests/golden/
    config2_fp16_storage_gap.txt, written from the oracle alone: the cell state grows by up to
    one per frame in this network and the two modes drift apart to 4e-2 by frame 40), twice
    that file's running maximum after that."""
    import os
    gap_file = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                            "config2_fp16_storage_gap.txt")
    gap = np.loadtxt(gap_file, comments="#")
    assert gap.shape[0] == 60 and np.array_equal(gap[:, 0], np.arange(60))
    frames = list(si.tool_scene_frames(60, 1080, 1920, 1))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    errs = _run_stream(hs, ctx, net=hs.HS_NET_RESNET18_CONVLSTM, net_name="resnet18_convlstm",
                       frames=frames, net_w=854, net_h=480, blob=blob, fp32_input=False,
                       check_state=True, tag="config2-60", emulate=False, storage_gap=gap[:, 1])
    assert len(errs) == 60


@pytest.mark.parametrize("fw,fh,nw,nh,thr,alpha", [
    (128, 128, 128, 128, 0.5, 0.0),      # identity resize, alpha 0 => overlay == input
    (322, 241, 96, 72, 0.75, 1.0),       # odd frame size (pitch padding), upscale-free, opaque
    (64, 48, 160, 120, 0.3, 0.37),       # upscaling resize, odd alpha
    (48, 8, 16384, 8, 0.5, 0.5),         # widest network input: interpolation weights up to 2^15
    (10922, 9, 128, 16, 0.5, 0.5),       # widest frame (32768-byte rows), 85x decimation
])
def test_tiny_net_edge_shapes(hs, ctx, fw, fh, nw, nh, thr, alpha):
    frames = list(si.uniform_frames(2, fh, fw, 5))
    blob = si.he_normal_blob(si.TINY4_LAYERS, 3)
    _run_stream(hs, ctx, net=hs.HS_NET_TINY4, net_name="tiny4", frames=frames, net_w=nw, net_h=nh,
                blob=blob, fp32_input=True, threshold=thr, alpha=alpha,
                tag=f"edge-{fw}x{fh}-{nw}x{nh}")
    if alpha == 0.0:
        pass  # check_frame already compared against the oracle overlay (== input for alpha 0)


@pytest.mark.parametrize("fw,fh,nw,nh,net_name,marker", [
    (320, 240, 128, 128, "tiny4", (12, 1, 2)),       # 10-pixel cells, markers of all 8 tools crowd
    (322, 241, 96, 72, "tiny4", (7, 0, 1)),          # ragged rows: byte path of the overlay
    (1920, 1080, 854, 480, "resnet18_convlstm", (12, 1, 2)),   # full size, coalesced path
    (640, 360, 288, 160, "resnet18_convlstm", (20, 3, 3)),     # thick marker, big labels, clipping
])
def test_annotation_layer_markers_and_labels(hs, ctx, fw, fh, nw, nh, net_name, marker):
    """Overlay with the annotation layer on: the frame must equal, bit for bit, the oracle's
    mask blend + markers + 'T<k>' labels drawn from the GPU's own argmax / present record."""
    tiny = net_name == "tiny4"
    frames = list(si.uniform_frames(2, fh, fw, 9)) if tiny else \
        list(si.tool_scene_frames(2, fh, fw, 9))
    blob = si.he_normal_blob(si.TINY4_LAYERS if tiny else si.RESNET18_CONVLSTM_LAYERS, 4)
    _run_stream(hs, ctx, net=hs.HS_NET_TINY4 if tiny else hs.HS_NET_RESNET18_CONVLSTM,
                net_name=net_name, frames=frames, net_w=nw, net_h=nh, blob=blob, fp32_input=tiny,
                glyphs=si.DEFAULT_GLYPHS, marker=marker, tag=f"annot-{fw}x{fh}")


def test_reset_state_and_queue_semantics(hs, ctx):
    from paper_2402_04466_amd.harness import AppStream
    frames = list(si.tool_scene_frames(2, 180, 320, 7))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=320, frame_h=180, net_w=160,
                  net_h=96, blob=blob, palette=PAL, queue_depth=2)
    try:
        assert s.poll() is None                                  # nothing submitted yet
        import os
        hs.hs_set_cpu_affinity(s.app, sorted(os.sched_getaffinity(0))[0])   # completion thread
        with pytest.raises(hs.HsError):
            hs.hs_set_cpu_affinity(s.app, 1 << 20)
        d_in = s.upload_frame(frames[0])
        outs = [s.new_output() for _ in range(3)]

        def one(i):
            assert s.submit(d_in, outs[i % 3], i) == hs.HS_OK
            return s.fetch(s.wait())["logits"]
        l0 = one(0)
        l1 = one(1)
        assert not np.array_equal(l0, l1)                        # state carried across frames
        hs.hs_reset_state(s.app)
        l2 = one(2)
        assert np.array_equal(l0, l2)                            # reset => same as first frame
        # queue_depth 2: a third unpolled frame is refused and not enqueued
        assert s.submit(d_in, outs[0], 10) == hs.HS_OK
        assert s.submit(d_in, outs[1], 11) == hs.HS_OK
        assert s.submit(d_in, outs[2], 12) == hs.HS_E_QUEUE_FULL
        assert s.wait().frame_id == 10 and s.wait().frame_id == 11
        assert s.poll() is None
        hs.hs_set_cpu_affinity(s.app, -1)
    finally:
        s.close()


@pytest.mark.parametrize("net,net_name,layers,fw,fh,nw,nh,fp32,seed", [
    ("HS_NET_RESNET18_CONVLSTM", "resnet18_convlstm", "RESNET18_CONVLSTM_LAYERS", 640, 360, 288, 160,
     False, 1),
    ("HS_NET_TINY4", "tiny4", "TINY4_LAYERS", 320, 240, 128, 128, True, 0),
])
def test_batched_streams_match_per_stream_oracles(hs, ctx, net, net_name, layers, fw, fh, nw, nh,
                                                  fp32, seed):
    """Cross-stream batched inference: 3 streams through ONE batched application (one shared
    weight copy, the network run once over the batch, ConvLSTM state per stream) against 3
    independent oracle streams, 3 frames each."""
    from paper_2402_04466_amd.harness import AppStream
    B, T = 3, 3
    blob = si.he_normal_blob(getattr(si, layers), seed)
    if net_name == "tiny4":
        frames = [list(si.uniform_frames(T, fh, fw, 20 + j)) for j in range(B)]
    else:
        frames = [list(si.tool_scene_frames(T, fh, fw, 20 + j)) for j in range(B)]
    s = AppStream(ctx, net=getattr(hs, net), frame_w=fw, frame_h=fh, net_w=nw, net_h=nh, blob=blob,
                  palette=PAL, queue_depth=2, net_fp32_input=fp32, batch=B)
    oracles = [make_oracles(net_name, blob, nw, nh, not fp32, PAL) for _ in range(B)]
    try:
        with pytest.raises(hs.HsError):                     # single-frame call on a batched app
            hs.hs_submit_frame(s.app, 256, 512, 0)
        for t in range(T):
            print(f"[batch-{net_name}] frame {t}", flush=True)
            d_in = [s.upload_frame(frames[j][t]) for j in range(B)]
            d_out = [s.new_output() for _ in range(B)]
            assert s.submit_batch(d_in, d_out, t) == hs.HS_OK
            rs = s.wait_batch()
            assert len(rs) == B and all(r.frame_id == t for r in rs)
            for j in range(B):
                g = s.fetch(rs[j], d_out[j])
                a, b = oracles[j][0].process(frames[j][t]), oracles[j][1].process(frames[j][t])
                check_frame(g, frames[j][t], a, b, threshold=0.5, alpha=0.5, palette=PAL,
                            fp32_input=fp32, tag=f"batch-{net_name}/stream{j}/frame{t}")
                if net_name != "tiny4":
                    gh, gc = s.state(rs[j], stream=j)
                    assert rms_rel(gh, a["h"]) <= TOL_STATE_RMS and rms_rel(gc, a["c"]) <= TOL_STATE_RMS
    finally:
        s.close()


def test_batch16_ragged_maps_on_the_large_grid_kernels(hs, ctx):
    """Sixteen streams of 640x360 frames batched through a 416x240 network input: feature maps of
    60x104, 30x52, 15x26 and 8x13 pixels, none a multiple of the 8 x 16 spatial tile, on grids
    large enough (512 workgroups in stage 2) for the kernels that only run from a few frames
    per launch on -- the tile-walking ones and the one that reads its weights as MFMA fragments
    straight from memory.  Streams 0, 9 and 15 against their own oracle streams over two
    frames, every stage; all sixteen finite and distinct."""
    from paper_2402_04466_amd.harness import AppStream
    B, T, sampled = 16, 2, (0, 9, 15)
    fw, fh, nw, nh = 640, 360, 416, 240
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 6)
    frames = {j: list(si.tool_scene_frames(T, fh, fw, 40 + j)) for j in range(B)}
    s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=fw, frame_h=fh, net_w=nw, net_h=nh,
                  blob=blob, palette=PAL, queue_depth=2, batch=B)
    oracles = {j: make_oracles("resnet18_convlstm", blob, nw, nh, True, PAL) for j in sampled}
    try:
        for t in range(T):
            print(f"[batch16-ragged] frame {t}", flush=True)
            d_in = [s.upload_frame(frames[j][t]) for j in range(B)]
            d_out = [s.new_output() for _ in range(B)]
            assert s.submit_batch(d_in, d_out, t) == hs.HS_OK
            rs = s.wait_batch()
            logits = [s.fetch(rs[j])["logits"] for j in range(B)]
            assert all(np.isfinite(l).all() for l in logits)
            for j in range(1, B):
                assert not np.array_equal(logits[j], logits[0])
            for j in sampled:
                g = s.fetch(rs[j], d_out[j])
                a, b = oracles[j][0].process(frames[j][t]), oracles[j][1].process(frames[j][t])
                check_frame(g, frames[j][t], a, b, threshold=0.5, alpha=0.5, palette=PAL,
                            fp32_input=False, tag=f"batch16-ragged/stream{j}/frame{t}")
                gh, gc = s.state(rs[j], stream=j)
                assert rms_rel(gh, a["h"]) <= TOL_STATE_RMS and rms_rel(gc, a["c"]) <= TOL_STATE_RMS
    finally:
        s.close()


def test_config5_full_size_batch12_sampled_streams(hs, ctx):
    """The saturation configuration as bench.py runs it: 12 streams of 1920x1080 frames batched
    through one pass of the big network (854x480 input, HIP-graph launch, the large-grid kernel
    variants), two frames with the state carried.  Streams 0, 7 and 11 are checked in full
    against their own oracle streams; all twelve must show distinct, finite outputs."""
    from paper_2402_04466_amd.harness import AppStream
    B, T, sampled = 12, 2, (0, 7, 11)
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    frames = {j: list(si.tool_scene_frames(T, 1080, 1920, 13 + j)) for j in range(B)}
    s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=1920, frame_h=1080, net_w=854,
                  net_h=480, blob=blob, palette=PAL, queue_depth=2, batch=B)
    oracles = {j: make_oracles("resnet18_convlstm", blob, 854, 480, True, PAL) for j in sampled}
    try:
        for t in range(T):
            print(f"[config5] frame {t}", flush=True)
            d_in = [s.upload_frame(frames[j][t]) for j in range(B)]
            d_out = [s.new_output() for _ in range(B)]
            assert s.submit_batch(d_in, d_out, t) == hs.HS_OK
            rs = s.wait_batch()
            assert len(rs) == B and all(r.frame_id == t for r in rs)
            logits = [s.fetch(rs[j])["logits"] for j in range(B)]
            assert all(np.isfinite(l).all() for l in logits)
            for j in range(1, B):
                assert not np.array_equal(logits[j], logits[0])       # streams are not mixed up
            for j in sampled:
                g = s.fetch(rs[j], d_out[j])
                a, b = oracles[j][0].process(frames[j][t]), oracles[j][1].process(frames[j][t])
                check_frame(g, frames[j][t], a, b, threshold=0.5, alpha=0.5, palette=PAL,
                            fp32_input=False, tag=f"config5/stream{j}/frame{t}")
                gh, gc = s.state(rs[j], stream=j)
                assert rms_rel(gh, a["h"]) <= TOL_STATE_RMS and rms_rel(gc, a["c"]) <= TOL_STATE_RMS
    finally:
        s.close()


@pytest.mark.parametrize("mode,depth", [("HS_LAUNCH_GRAPH", 4), ("HS_LAUNCH_EAGER", 4),
                                        ("HS_LAUNCH_GRAPH", 2), ("HS_LAUNCH_GRAPH", 3),
                                        ("HS_LAUNCH_EAGER", 2), ("HS_LAUNCH_EAGER", 3)])
def test_back_to_back_frames_overlap_and_match_one_at_a_time(hs, ctx, mode, depth):
    """Consecutive frames of one stream run in two lanes and may overlap on the GPU; only the
    recurrent cell chains them.  Eight frames submitted as fast as the queue takes them must give,
    frame by frame and bit for bit, what the same frames give when each is waited for before the
    next is submitted, and the same final recurrent state."""
    from paper_2402_04466_amd.harness import AppStream
    T = 8
    frames = list(si.tool_scene_frames(T, 360, 640, 17))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 2)
    # depth 3: an odd queue cannot alternate lanes strictly and runs in a single lane
    s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=640, frame_h=360, net_w=288,
                  net_h=160, blob=blob, palette=PAL, queue_depth=depth)
    hs.hs_set_launch_mode(s.app, getattr(hs, mode))
    try:
        d_in = [s.upload_frame(f) for f in frames]
        d_out = [s.new_output() for _ in range(T)]
        ref = []
        for t in range(T):                                   # one at a time
            assert s.submit(d_in[t], d_out[t], t) == hs.HS_OK
            r = s.wait()
            ref.append(s.fetch(r, d_out[t]))
        ref_h, ref_c = s.state(r)
        ref_x = s.features(r)
        hs.hs_reset_state(s.app)
        for o in d_out:
            o.zero_()
        torch.cuda.synchronize()
        got, sub = [], 0
        while len(got) < T:                                   # as fast as the queue takes them
            while sub < T and s.submit(d_in[sub], d_out[sub], sub) == hs.HS_OK:
                sub += 1
            r = s.wait()
            assert r.frame_id == len(got)
            got.append(s.fetch(r, d_out[len(got)]))
        for t in range(T):
            for k in ("logits", "mask", "argmax_idx", "overlay"):
                assert np.array_equal(ref[t][k], got[t][k]), f"frame {t}: {k} differs"
        h, c = s.state(r)
        assert np.array_equal(h, ref_h) and np.array_equal(c, ref_c)
        assert np.array_equal(s.features(r), ref_x)
    finally:
        s.close()


def test_long_back_to_back_run_is_deterministic(hs, ctx):
    """96 frames as fast as the queue takes them, twice from a reset state: every frame's logits
    and the final recurrent state must repeat exactly (no race between overlapping frames)."""
    from paper_2402_04466_amd.harness import AppStream
    T = 96
    frames = list(si.tool_scene_frames(8, 360, 640, 23))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 3)
    s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=640, frame_h=360, net_w=288,
                  net_h=160, blob=blob, palette=PAL, queue_depth=4)
    try:
        d_in = [s.upload_frame(f) for f in frames]
        d_out = [s.new_output() for _ in range(4)]

        def run():
            got, sub = [], 0
            while len(got) < T:
                while sub < T and s.submit(d_in[sub % 8], d_out[sub % 4], sub) == hs.HS_OK:
                    sub += 1
                r = s.wait()
                assert r.frame_id == len(got)
                got.append(s.fetch(r)["logits"].copy())
            return got, s.state(r)
        a, (ha, ca) = run()
        hs.hs_reset_state(s.app)
        b, (hb, cb) = run()
        for t in range(T):
            assert np.array_equal(a[t], b[t]), f"frame {t} differs between the two runs"
        assert np.array_equal(ha, hb) and np.array_equal(ca, cb)
        assert not np.array_equal(a[0], a[8])     # same input, different state: the cell is live
    finally:
        s.close()


def test_graph_and_kernel_by_kernel_launch_paths_agree(hs, ctx):
    """The pre-built HIP graph of stages 1-3 is replayed for several frames (with the host's
    own synchronisation and read-backs between replays) and must give, frame by frame and
    bit for bit, what the kernel-by-kernel path gives, state included."""
    from paper_2402_04466_amd.harness import AppStream
    frames = list(si.tool_scene_frames(5, 360, 640, 11))
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    kw = dict(net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=640, frame_h=360, net_w=288, net_h=160,
              blob=blob, palette=PAL, queue_depth=2)
    a, b = AppStream(ctx, **kw), AppStream(ctx, **kw)
    try:
        hs.hs_set_launch_mode(a.app, hs.HS_LAUNCH_GRAPH)
        hs.hs_set_launch_mode(b.app, hs.HS_LAUNCH_EAGER)
        for i, f in enumerate(frames):
            outs = []
            for s in (a, b):
                d_in, d_out = s.upload_frame(f), s.new_output()
                assert s.submit(d_in, d_out, i) == hs.HS_OK
                r = s.wait()
                assert r.t_submit_ns <= r.t_enqueued_ns
                assert r.t_submit_ns <= r.t_pre_done_ns <= r.t_infer_done_ns <= r.t_post_done_ns \
                    <= r.t_overlay_done_ns
                g = s.fetch(r, d_out)
                g["h"], g["c"] = s.state(r)
                outs.append(g)
            for k in outs[0]:
                assert np.array_equal(outs[0][k], outs[1][k]), (i, k)
    finally:
        a.close()
        b.close()


def test_partition_admission_and_masked_results_identical(hs, ctx):
    """Two applications on disjoint CU sets; an overlapping request is refused and changes
    nothing; results under a CU mask equal the unpartitioned ones bit for bit."""
    from paper_2402_04466_amd.harness import AppStream
    n_cus = hs.hs_device_cus(ctx)
    assert n_cus >= 64
    frames = list(si.uniform_frames(1, 240, 320, 9))
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    kw = dict(net=hs.HS_NET_TINY4, frame_w=320, frame_h=240, net_w=128, net_h=128, blob=blob,
              palette=PAL, queue_depth=2, net_fp32_input=True)
    a, b = AppStream(ctx, **kw), AppStream(ctx, **kw)
    try:
        d_in, o1, o2 = a.upload_frame(frames[0]), a.new_output(), a.new_output()
        assert a.submit(d_in, o1, 0) == hs.HS_OK
        ref = a.fetch(a.wait(), o1)
        half = n_cus // 2
        hs.hs_set_partition(a.app, hs.cu_mask_words(range(0, half - 8)),
                            hs.cu_mask_words(range(half - 8, half)))
        with pytest.raises(hs.HsError) as ei:                   # overlaps a's claim
            hs.hs_set_partition(b.app, hs.cu_mask_words(range(half - 4, n_cus)),
                                hs.cu_mask_words(range(half - 4, n_cus)))
        assert ei.value.status == hs.HS_E_OVERSUBSCRIBED
        if n_cus < 256:                                          # CU the device does not have
            with pytest.raises(hs.HsError):
                hs.hs_set_partition(b.app, hs.cu_mask_words([n_cus]), hs.cu_mask_words([n_cus]))
        with pytest.raises(hs.HsError) as ei:                    # empty overlay mask
            hs.hs_set_partition(b.app, hs.cu_mask_words(range(half, n_cus)), hs.cu_mask_words([]))
        assert ei.value.status == hs.HS_E_OVERSUBSCRIBED
        # a mask that leaves an XCD without a CU (CU i is on XCD i mod 8) is refused, whichever
        # of the two masks it is, and b stays unpartitioned and usable
        free = list(range(half, n_cus))
        no_xcd3 = [c for c in free if c % (n_cus // 32) != 3]
        for mi, mo in ((no_xcd3, free), (free, no_xcd3), (free[:7], free[:7])):
            with pytest.raises(hs.HsError) as ei:
                hs.hs_set_partition(b.app, hs.cu_mask_words(mi), hs.cu_mask_words(mo))
            assert ei.value.status == hs.HS_E_INVAL and "XCD" in str(ei.value)
        hs.hs_set_partition(b.app, hs.cu_mask_words(range(half, n_cus)),
                            hs.cu_mask_words(range(half, n_cus)))
        assert a.submit(d_in, o2, 1) == hs.HS_OK
        got = a.fetch(a.wait(), o2)
        for k in ("logits", "mask", "overlay", "net_input"):
            assert np.array_equal(ref[k], got[k]), k
        d_in_b, ob = b.upload_frame(frames[0]), b.new_output()
        assert b.submit(d_in_b, ob, 0) == hs.HS_OK
        got_b = b.fetch(b.wait(), ob)
        assert np.array_equal(ref["logits"], got_b["logits"])
        assert np.array_equal(ref["overlay"], got_b["overlay"])
        hs.hs_set_partition(a.app, None, None)                   # release: b may now take them
        hs.hs_set_partition(b.app, hs.cu_mask_words(range(0, n_cus)),
                            hs.cu_mask_words(range(0, n_cus)))
    finally:
        a.close()
        b.close()


def test_device_copy_kernel(hs, ctx):
    """The plain copy kernel that byte counters are calibrated against: exact, ragged sizes too."""
    for nbytes in (16, 4096 + 16, 3 * 1024 * 1024 + 48):
        a = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda:0")
        b = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        hs.hs_device_copy(ctx, b.data_ptr(), a.data_ptr(), nbytes)
        torch.cuda.synchronize()
        assert torch.equal(b[:nbytes], a) and int(b[nbytes:].sum()) == 0
    with pytest.raises(hs.HsError):
        hs.hs_device_copy(ctx, 256, 512, 24)          # not a multiple of 16


def test_partition_copy_runs_under_the_application_mask(hs, ctx):
    """The masked copy that gives a partition's bandwidth denominator: exact, and a 16-CU
    partition moves the same bytes more slowly than the whole device."""
    from paper_2402_04466_amd.harness import AppStream
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    a = AppStream(ctx, net=hs.HS_NET_TINY4, frame_w=320, frame_h=240, net_w=128, net_h=128,
                  blob=blob, palette=PAL, queue_depth=2)
    try:
        nbytes = 64 << 20
        src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda:0")
        dst = torch.zeros_like(src)
        torch.cuda.synchronize()
        t_all = hs.hs_partition_copy(a.app, dst.data_ptr(), src.data_ptr(), nbytes, 5)
        assert torch.equal(dst, src) and t_all > 0
        dst.zero_()
        torch.cuda.synchronize()
        hs.hs_set_partition(a.app, hs.cu_mask_words(range(16)), hs.cu_mask_words(range(16)))
        t_16 = hs.hs_partition_copy(a.app, dst.data_ptr(), src.data_ptr(), nbytes, 5)
        assert torch.equal(dst, src)
        print(f"[partition copy] all CUs {2 * nbytes / t_all / 1e9:.0f} GB/s, "
              f"16 CUs {2 * nbytes / t_16 / 1e9:.0f} GB/s", flush=True)
        assert t_16 > 1.5 * t_all
        with pytest.raises(hs.HsError):
            hs.hs_partition_copy(a.app, dst.data_ptr(), src.data_ptr(), 24, 1)
    finally:
        a.close()


def test_kernel_timing_reports_every_family(hs, ctx):
    from paper_2402_04466_amd.harness import AppStream
    frames = list(si.uniform_frames(1, 240, 320, 2))
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    s = AppStream(ctx, net=hs.HS_NET_TINY4, frame_w=320, frame_h=240, net_w=128, net_h=128,
                  blob=blob, palette=PAL, queue_depth=2)
    try:
        hs.hs_set_kernel_timing(s.app, True)
        d_in, d_out = s.upload_frame(frames[0]), s.new_output()
        for i in range(3):
            assert s.submit(d_in, d_out, i) == hs.HS_OK
            s.wait()
        t = {e["name"]: e for e in hs.hs_get_kernel_times(s.app)}
        assert {"resize_norm", "conv_mfma", "postprocess", "overlay"} <= set(t)
        assert t["conv_mfma"]["launches"] == 12 and t["conv_mfma"]["total_ms"] > 0
        assert abs(t["conv_mfma"]["flops"] / 3 - 36.6e6) < 0.5e6     # 36.6 MFLOP per frame
    finally:
        s.close()


@pytest.mark.parametrize("partition", ["none", "shared", "split"])
def test_concurrent_paced_streams_match_solo_runs(hs, ctx, partition):
    """Configurations 3 and 4 in the way the benchmark drives them: several applications, one
    submitting thread each, paced at a fixed rate and overlapping on the GPU, unpartitioned or
    on disjoint CU sets (one stream per partition, or inference / overlay on separate sets).
    Every frame of every stream must equal, bit for bit, what the same application computes
    when it runs alone (the recurrent state makes frame k depend on frames 0..k-1), and the
    first frame is checked against the oracle."""
    from paper_2402_04466_amd.harness import AppStream, run_paced
    fw, fh = 640, 360
    specs = [("resnet18_convlstm", hs.HS_NET_RESNET18_CONVLSTM, si.RESNET18_CONVLSTM_LAYERS, 224, 128),
             ("tiny4", hs.HS_NET_TINY4, si.TINY4_LAYERS, 128, 128),
             ("resnet18_convlstm", hs.HS_NET_RESNET18_CONVLSTM, si.RESNET18_CONVLSTM_LAYERS, 160, 96),
             ("tiny4", hs.HS_NET_TINY4, si.TINY4_LAYERS, 96, 64)]
    n_frames = depth = 12      # one queue slot per frame: every frame's buffers stay readable
    n_cus = hs.hs_device_cus(ctx)
    apps, frames, blobs = [], [], []
    try:
        for i, (name, net, layers, nw, nh) in enumerate(specs):
            blob = si.he_normal_blob(layers, 10 + i)
            blobs.append(blob)
            apps.append(AppStream(ctx, net=net, frame_w=fw, frame_h=fh, net_w=nw, net_h=nh,
                                  blob=blob, palette=PAL, queue_depth=depth))
            frames.append([apps[-1].upload_frame(f)
                           for f in si.tool_scene_frames(n_frames, fh, fw, 60 + i)])
        host_frames = [list(si.tool_scene_frames(1, fh, fw, 60 + i))[0] for i in range(len(specs))]
        # solo reference: one application at a time, one frame at a time
        solo = []
        for a, fr in zip(apps, frames):
            per = []
            for k, d_in in enumerate(fr):
                o = a.new_output()
                assert a.submit(d_in, o, k) == hs.HS_OK
                per.append(a.fetch(a.wait(), o))
            solo.append(per)
            hs.hs_reset_state(a.app)
        if partition != "none":
            per_app = (n_cus // 8 // len(apps)) * 8
            for i, a in enumerate(apps):
                cus = list(range(i * per_app, (i + 1) * per_app))
                ci, co = (cus, cus) if partition == "shared" else (cus[:-8], cus[-8:])
                hs.hs_set_partition(a.app, hs.cu_mask_words(ci), hs.cu_mask_words(co))
        outs = [[[a.new_output()] for _ in range(n_frames)] for a in apps]
        print(f"[concurrent {partition}] {len(apps)} applications x {n_frames} frames", flush=True)
        results, dropped = run_paced(apps, [[[t] for t in fr] for fr in frames], 2000.0, outs)
        assert sum(dropped) == 0
        for i, (a, rs) in enumerate(zip(apps, results)):
            assert [r[0].frame_id for r in rs] == list(range(n_frames))
            for k, r in enumerate(rs):
                g = a.fetch(r[0], outs[i][k][0])
                for key in ("net_input", "logits", "heat", "mask", "argmax_idx", "present", "overlay"):
                    assert np.array_equal(g[key], solo[i][k][key]), (partition, i, k, key)
        for i, (name, net, layers, nw, nh) in enumerate(specs):
            o32, _ = make_oracles(name, blobs[i], nw, nh, True, PAL)
            check_frame(solo[i][0], host_frames[i], o32.process(host_frames[i]), None,
                        threshold=0.5, alpha=0.5, palette=PAL, fp32_input=False,
                        tag=f"concurrent/{i}")
    finally:
        for a in apps:
            a.close()


def _equal_partitions(n_cus, n_apps, split):
    """n_apps disjoint CU sets of equal size out of groups of 8 consecutive CUs (one CU per
    XCD each), two groups left unclaimed; split: the last group of a set serves the overlay."""
    per = (n_cus // 8 - 2) // n_apps
    parts = []
    for i in range(n_apps):
        cus = list(range(i * per * 8, (i + 1) * per * 8))
        parts.append((cus[:-8], cus[-8:]) if split else (cus, cus))
    return parts


@pytest.mark.parametrize("n_apps,first_seed", [(5, 2), (6, 7)])
def test_configs_3_and_4_full_size_concurrent_applications(hs, ctx, n_apps, first_seed):
    """Configurations 3 and 4 at configuration size: five (seeds 2-6) and six (seeds 7-12)
    applications of the 1920x1080 -> 854x480 ResNet-18-style + ConvLSTM network, every stream
    paced at 60 frames per second by the library's driver, one submitting thread each --
    unpartitioned, on equal CU partitions with one queue each, and on equal partitions with
    inference and overlay on separate CU sets (the paper's Section IV-A / IV-B arrangement).
    In each arrangement every frame of every stream must equal, bit for bit, what the same
    application computes alone (frame k depends on frames 0..k-1 through the cell state); the
    first and the last frame of every stream are checked against the oracle."""
    from paper_2402_04466_amd.harness import AppStream, run_paced
    fw, fh, nw, nh, n_frames = 1920, 1080, 854, 480, 4
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    n_cus = hs.hs_device_cus(ctx)
    keys = ("net_input", "logits", "heat", "mask", "argmax_idx", "present", "peak", "overlay")
    apps, d_frames, host_frames = [], [], []
    try:
        for i in range(n_apps):
            a = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=fw, frame_h=fh, net_w=nw,
                          net_h=nh, blob=blob, palette=PAL, queue_depth=n_frames)
            apps.append(a)
            host_frames.append(list(si.tool_scene_frames(n_frames, fh, fw, first_seed + i)))
            d_frames.append([a.upload_frame(f) for f in host_frames[-1]])
        solo = []
        for i, a in enumerate(apps):
            print(f"[configs-3-4 {n_apps} apps] solo run of stream {i}", flush=True)
            per = []
            for k, d_in in enumerate(d_frames[i]):
                o = a.new_output()
                assert a.submit(d_in, o, k) == hs.HS_OK
                per.append(a.fetch(a.wait(), o))
            solo.append(per)
        outs = [[[a.new_output()] for _ in range(n_frames)] for a in apps]
        for arrangement in ("unpartitioned", "shared", "split"):
            for i, a in enumerate(apps):
                hs.hs_reset_state(a.app)
            if arrangement != "unpartitioned":
                parts = _equal_partitions(n_cus, n_apps, arrangement == "split")
                for a in apps:                       # release first: the new sets overlap old ones
                    hs.hs_set_partition(a.app, None, None)
                for a, (ci, co) in zip(apps, parts):
                    hs.hs_set_partition(a.app, hs.cu_mask_words(ci), hs.cu_mask_words(co))
            for per_app in outs:
                for o in per_app:
                    o[0].zero_()
            torch.cuda.synchronize()
            print(f"[configs-3-4 {n_apps} apps] {arrangement}: {n_frames} frames per stream at "
                  f"60 fps", flush=True)
            results, dropped = run_paced(apps, [[[t] for t in fr] for fr in d_frames], 60.0, outs)
            assert sum(dropped) == 0
            for i, (a, rs) in enumerate(zip(apps, results)):
                assert [r[0].frame_id for r in rs] == list(range(n_frames))
                for k, r in enumerate(rs):
                    assert r[0].t_submit_ns <= r[0].t_pre_done_ns <= r[0].t_infer_done_ns \
                        <= r[0].t_post_done_ns <= r[0].t_overlay_done_ns
                    g = a.fetch(r[0], outs[i][k][0])
                    for key in keys:
                        assert np.array_equal(g[key], solo[i][k][key]), (arrangement, i, k, key)
        for i in range(n_apps):
            print(f"[configs-3-4 {n_apps} apps] oracle for stream {i}", flush=True)
            o32, _ = make_oracles("resnet18_convlstm", blob, nw, nh, True, PAL)
            for k, f in enumerate(host_frames[i]):
                ref = o32.process(f)
                if k in (0, n_frames - 1):
                    check_frame(solo[i][k], f, ref, None, threshold=0.5, alpha=0.5, palette=PAL,
                                fp32_input=False, tag=f"configs-3-4/{n_apps}/stream{i}/frame{k}")
    finally:
        for a in apps:
            a.close()


def test_mux_refuses_a_wrong_batch_and_group_members(hs, ctx):
    """hs_create_mux sizes its buffers by `batch` and hands them to the batch calls of the
    application: a batch that is not the application's is HS_E_INVAL, a member of a group
    HS_E_STATE (it is driven through the group only)."""
    from paper_2402_04466_amd import api
    from paper_2402_04466_amd.harness import AppStream, GroupStream
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    kw = dict(net=hs.HS_NET_TINY4, frame_w=320, frame_h=240, net_w=128, net_h=128, blob=blob,
              palette=PAL, queue_depth=2)
    a3, a1, b1 = AppStream(ctx, batch=3, **kw), AppStream(ctx, **kw), AppStream(ctx, **kw)
    g = None
    try:
        for wrong in (1, 2, 4, 16):
            with pytest.raises(hs.HsError) as ei:
                api.hs_create_mux(a3.app, wrong)
            assert ei.value.status == hs.HS_E_INVAL and "batches 3" in str(ei.value)
        with pytest.raises(hs.HsError) as ei:
            api.hs_create_mux(a1.app, 2)
        assert ei.value.status == hs.HS_E_INVAL
        api.hs_destroy_mux(api.hs_create_mux(a3.app, 3))
        g = GroupStream(ctx, [a1, b1])
        with pytest.raises(hs.HsError) as ei:
            api.hs_create_mux(a1.app, 1)
        assert ei.value.status == hs.HS_E_STATE
    finally:
        if g is not None:
            g.close()
        else:
            a1.close()
            b1.close()
        a3.close()


def test_create_destroy_cycles_release_everything(hs, ctx):
    """Applications (partitioned or not, grouped, behind a mux) can be created and destroyed
    many times over: streams, events, threads and CU claims are all returned."""
    from paper_2402_04466_amd import api
    from paper_2402_04466_amd.harness import AppStream, GroupStream
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    frame = si.uniform_frames(1, 240, 320, 3)[0]
    n_cus = hs.hs_device_cus(ctx)
    ref = None
    for cycle in range(24):
        kw = dict(net=hs.HS_NET_TINY4, frame_w=320, frame_h=240, net_w=128, net_h=128, blob=blob,
                  palette=PAL, queue_depth=2 + cycle % 3)
        a, b = AppStream(ctx, **kw), AppStream(ctx, **kw)
        if cycle % 2:
            hs.hs_set_partition(a.app, hs.cu_mask_words(range(0, n_cus // 2)),
                                hs.cu_mask_words(range(0, n_cus // 2)))
            hs.hs_set_partition(b.app, hs.cu_mask_words(range(n_cus // 2, n_cus - 8)),
                                hs.cu_mask_words(range(n_cus - 8, n_cus)))
        d_in, d_out = a.upload_frame(frame), a.new_output()
        if cycle % 3 == 0:
            g = GroupStream(ctx, [a, b])
            assert g.submit(d_in, d_out, cycle) == hs.HS_OK
            rs = g.wait_batch()
            got = a.fetch(rs[0])["logits"]
            g.close()
        else:
            mux = api.hs_create_mux(a.app, 1)
            assert api.hs_mux_submit(mux, 0, d_in.data_ptr(), d_out.data_ptr(), cycle) == hs.HS_OK
            r = api.hs_mux_wait(mux, 0)
            got = a.fetch(r)["logits"]
            api.hs_destroy_mux(mux)
            a.close()
            b.close()
        ref = got if ref is None else ref
        assert np.array_equal(got, ref), cycle


def test_long_concurrent_back_to_back_runs_are_deterministic(hs, ctx):
    """Five applications of different kinds, sizes and queue depths push 400 frames each through
    the device at the same time, as fast as their queues take them (native driver, one thread
    each, frames of one application overlapping in two lanes where its depth is even).  Twice
    over the final outputs -- which depend on every earlier frame through the recurrent state --
    must be identical, and identical to what each application reaches when it runs alone."""
    from paper_2402_04466_amd.harness import AppStream, run_back_to_back
    fw, fh, n = 640, 360, 400
    specs = [(hs.HS_NET_RESNET18_CONVLSTM, si.RESNET18_CONVLSTM_LAYERS, 224, 128, 4),
             (hs.HS_NET_TINY4, si.TINY4_LAYERS, 128, 128, 4),
             (hs.HS_NET_RESNET18_CONVLSTM, si.RESNET18_CONVLSTM_LAYERS, 288, 160, 2),
             (hs.HS_NET_RESNET18_CONVLSTM, si.RESNET18_CONVLSTM_LAYERS, 160, 96, 3),
             (hs.HS_NET_TINY4, si.TINY4_LAYERS, 96, 64, 6)]
    apps, frames, outs = [], [], []
    try:
        for i, (net, layers, nw, nh, depth) in enumerate(specs):
            a = AppStream(ctx, net=net, frame_w=fw, frame_h=fh, net_w=nw, net_h=nh,
                          blob=si.he_normal_blob(layers, 20 + i), palette=PAL, queue_depth=depth)
            apps.append(a)
            frames.append([[a.upload_frame(f)] for f in si.tool_scene_frames(7, fh, fw, 80 + i)])
            outs.append([[a.new_output()] for _ in range(depth)])

        def last_outputs(results):
            got = []
            for a, rs in zip(apps, results):
                assert [r[0].frame_id for r in rs] == list(range(n))
                g = a.fetch(rs[-1][0])
                got.append((g["logits"].copy(), g["mask"].copy()))
            return got

        runs = []
        for rep in range(2):
            for a in apps:
                hs.hs_reset_state(a.app)
            print(f"[long concurrent] pass {rep}: {len(apps)} applications x {n} frames", flush=True)
            results, _ = run_back_to_back(apps, frames, outs, n)
            runs.append(last_outputs(results))
        for i in range(len(apps)):
            assert np.array_equal(runs[0][i][0], runs[1][i][0]), f"application {i}: passes differ"
            assert np.array_equal(runs[0][i][1], runs[1][i][1]), f"application {i}: passes differ"
        for i, a in enumerate(apps):
            hs.hs_reset_state(a.app)
            results, _ = run_back_to_back([a], [frames[i]], [outs[i]], n)
            g = a.fetch(results[0][-1][0])
            assert np.array_equal(g["logits"], runs[0][i][0]), f"application {i}: differs from solo"
    finally:
        for a in apps:
            a.close()


def test_submit_behind_a_producer_event(hs, ctx):
    """A frame still being written on the caller's own stream: with the producer's event handed
    to the submit, stage 1 waits for it on the GPU and sees the finished frame."""
    from paper_2402_04466_amd import api
    from paper_2402_04466_amd.harness import AppStream
    if not hasattr(torch.cuda, "_sleep"):
        pytest.skip("needs torch.cuda._sleep to hold the producer stream back")
    fw, fh = 640, 360
    frame = list(si.tool_scene_frames(1, fh, fw, 33))[0]
    blob = si.he_normal_blob(si.TINY4_LAYERS, 5)
    a = AppStream(ctx, net=hs.HS_NET_TINY4, frame_w=fw, frame_h=fh, net_w=128, net_h=128, blob=blob,
                  palette=PAL, queue_depth=2)
    try:
        ready = a.upload_frame(frame)
        d_out = a.new_output()
        assert a.submit(ready, d_out, 0) == hs.HS_OK
        ref = a.fetch(a.wait(), d_out)
        # the producer: a long spin, then the copy of the real frame over a zeroed buffer
        late = torch.zeros_like(ready)
        d_out2 = a.new_output()
        side = torch.cuda.Stream()
        ev = torch.cuda.Event()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            torch.cuda._sleep(200_000_000)             # ~0.1 s of GPU time on the side stream
            late.copy_(ready)
            ev.record(side)
        assert api.hs_submit_batch_after(a.app, [late.data_ptr()], [d_out2.data_ptr()], 1,
                                         ev.cuda_event) == hs.HS_OK
        r = a.wait()
        got = a.fetch(r, d_out2)
        for key in ("net_input", "logits", "mask", "overlay"):
            assert np.array_equal(got[key], ref[key]), key
        assert (r.t_overlay_done_ns - r.t_submit_ns) > 20_000_000   # it did wait for the producer
    finally:
        a.close()
