"""hs_submit_frame_static_scratch (the entry point for callers that cannot allocate: its
split-K scratch is a fixed device array inside the library) against hs_submit_frame, through
the C ABI: every output of every stage must be the same, bit for bit, on two calls in a row,
the second on a smaller input that leaves most of the array holding the first call's values."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _both_ways(hs, ctx, fw, fh, nw, nh, seed, tag):
    """Two frames (state carried) through the ordinary call, then, from a zeroed state, through
    the static-scratch call.  Returns the two lists of fetched outputs and the stream (open)."""
    from paper_2402_04466_amd.harness import AppStream
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=fw, frame_h=fh, net_w=nw,
                  net_h=nh, blob=blob, palette=si.DEFAULT_PALETTE, queue_depth=2)
    frames = [s.upload_frame(f) for f in si.tool_scene_frames(2, fh, fw, seed)]
    got = {}
    for name, call in (("workspace", hs.hs_submit_frame),
                       ("static", hs.hs_submit_frame_static_scratch)):
        hs.hs_reset_state(s.app)
        got[name] = []
        for k, d_in in enumerate(frames):
            print(f"[{tag}] {name} scratch, frame {k} {fw}x{fh} -> {nw}x{nh}", flush=True)
            d_out = s.new_output()
            assert call(s.app, d_in.data_ptr(), d_out.data_ptr(), k) == hs.HS_OK
            r = s.wait()
            assert r.frame_id == k
            g = s.fetch(r, d_out)
            g["h"], g["c"] = s.state(r)
            got[name].append(g)
    return got, s


def _assert_same(got, tag):
    for k, (a, b) in enumerate(zip(got["workspace"], got["static"])):
        assert np.abs(a["logits"]).max() > 0, f"{tag}: frame {k} computed nothing"
        for key in ("net_input", "logits", "heat", "mask", "argmax_idx", "present", "peak",
                    "overlay", "h", "c"):
            assert np.array_equal(a[key], b[key]), f"{tag}: frame {k}: {key} differs"


def test_static_scratch_submit_matches_workspace_submit_twice_in_a_row(hs):
    ctx = hs.hs_init(0)
    try:
        big, s_big = _both_ways(hs, ctx, 1920, 1080, 854, 480, 41, "no-alloc/1080p")
        try:
            _assert_same(big, "no-alloc/1080p")
            # second call in a row: a smaller input, the array still full of the first one's sums
            small, s_small = _both_ways(hs, ctx, 640, 360, 288, 160, 42, "no-alloc/360p")
            try:
                _assert_same(small, "no-alloc/360p")
                # one frame at a time: a second frame beside one in flight is refused, not raced
                d_in = s_big.upload_frame(next(iter(si.tool_scene_frames(1, 1080, 1920, 43))))
                outs = [s_big.new_output(), s_big.new_output()]
                torch.cuda.synchronize()
                assert hs.hs_submit_frame_static_scratch(s_big.app, d_in.data_ptr(),
                                                         outs[0].data_ptr(), 7) == hs.HS_OK
                try:
                    st = hs.hs_submit_frame_static_scratch(s_big.app, d_in.data_ptr(),
                                                           outs[1].data_ptr(), 8)
                    # the first frame may already have finished on a fast device: then it is taken
                    assert st == hs.HS_OK
                    second = True
                except hs.HsError as e:
                    assert e.status == hs.HS_E_STATE
                    second = False
                assert s_big.wait().frame_id == 7
                if second:
                    assert s_big.wait().frame_id == 8
            finally:
                s_small.close()
        finally:
            s_big.close()
    finally:
        hs.hs_shutdown(ctx)


def test_static_scratch_submit_refuses_what_it_cannot_serve(hs):
    """Batched applications and applications whose split-K scratch exceeds the fixed array are
    refused with a clear status; nothing is enqueued."""
    from paper_2402_04466_amd.harness import AppStream
    ctx = hs.hs_init(0)
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    try:
        # batch 2: HS_E_STATE
        s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=640, frame_h=360, net_w=288,
                      net_h=160, blob=blob, palette=si.DEFAULT_PALETTE, queue_depth=2, batch=2)
        try:
            d_in, d_out = s.new_output(), s.new_output()
            with pytest.raises(hs.HsError) as ei:
                hs.hs_submit_frame_static_scratch(s.app, d_in.data_ptr(), d_out.data_ptr(), 0)
            assert ei.value.status == hs.HS_E_STATE
        finally:
            s.close()
        # 1410 x 1488 network input: a 45 x 47 map, whose gate pre-activations alone (2115 pixels x
        # 1024 channels x 4 bytes = 8.66 MB) exceed the 8 MiB array: HS_E_NOMEM
        s = AppStream(ctx, net=hs.HS_NET_RESNET18_CONVLSTM, frame_w=1920, frame_h=1080,
                      net_w=1410, net_h=1488, blob=blob, palette=si.DEFAULT_PALETTE, queue_depth=2)
        try:
            d_in, d_out = s.new_output(), s.new_output()
            with pytest.raises(hs.HsError) as ei:
                hs.hs_submit_frame_static_scratch(s.app, d_in.data_ptr(), d_out.data_ptr(), 0)
            assert ei.value.status == hs.HS_E_NOMEM and "8388608" in str(ei.value)
            # the ordinary call still serves it
            assert hs.hs_submit_frame(s.app, d_in.data_ptr(), d_out.data_ptr(), 0) == hs.HS_OK
            assert s.wait().frame_id == 0
        finally:
            s.close()
    finally:
        hs.hs_shutdown(ctx)
