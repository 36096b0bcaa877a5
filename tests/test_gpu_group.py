"""GPU parity of multi-network applications (paper Section III-B): members run side by side on
the same frame, one overlay launch composites their layers.  Every member is checked stage by
stage against its own oracle; the shared picture is checked bit-exactly against the oracle's
layer compositing fed with the GPU's own masks / argmax (stage-isolated, as for single
applications) and, within the logit tolerance band, against the all-oracle picture."""
import numpy as np
import pytest

import synth_inputs as si
import oracle
from gpu_common import check_frame, make_oracles

pytestmark = pytest.mark.gpu
PAL_A = si.DEFAULT_PALETTE
PAL_B = si.DEFAULT_PALETTE[::-1].copy()
PAL_C = np.roll(si.DEFAULT_PALETTE, 3, axis=0).copy()
TINY = si.TINY4_LAYERS
RESNET = si.RESNET18_CONVLSTM_LAYERS


@pytest.fixture(scope="module")
def ctx(hs):
    c = hs.hs_init(0)
    yield c
    hs.hs_shutdown(c)


def _specs(fw, fh):
    """Three different networks on one frame: different kinds, input sizes, map sizes, colours,
    opacities, thresholds; two of them with annotations."""
    return [
        dict(net="HS_NET_TINY4", name="tiny4", layers=TINY, seed=0, nw=128, nh=128, pal=PAL_A,
             alpha=0.5, thr=0.5, glyphs=si.DEFAULT_GLYPHS, marker=(10, 1, 2)),
        dict(net="HS_NET_RESNET18_CONVLSTM", name="resnet18_convlstm", layers=RESNET, seed=1,
             nw=224, nh=128, pal=PAL_B, alpha=0.25, thr=0.5, glyphs=None, marker=(12, 1, 2)),
        dict(net="HS_NET_TINY4", name="tiny4", layers=TINY, seed=2, nw=96, nh=64, pal=PAL_C,
             alpha=0.75, thr=0.6, glyphs=si.DEFAULT_GLYPHS, marker=(6, 0, 1)),
    ]


def _build(hs, ctx, specs, fw, fh, depth):
    from paper_2402_04466_amd.harness import AppStream, GroupStream
    members, oracles = [], []
    for sp in specs:
        blob = si.he_normal_blob(sp["layers"], sp["seed"])
        members.append(AppStream(ctx, net=getattr(hs, sp["net"]), frame_w=fw, frame_h=fh,
                                 net_w=sp["nw"], net_h=sp["nh"], blob=blob, palette=sp["pal"],
                                 queue_depth=depth, threshold=sp["thr"], alpha=sp["alpha"],
                                 glyphs=sp["glyphs"], marker_arm=sp["marker"][0],
                                 marker_half=sp["marker"][1], glyph_scale=sp["marker"][2]))
        kw = dict(threshold=sp["thr"], alpha=sp["alpha"], glyphs=sp["glyphs"],
                  marker_arm=sp["marker"][0], marker_half=sp["marker"][1],
                  glyph_scale=sp["marker"][2])
        oracles.append(make_oracles(sp["name"], blob, sp["nw"], sp["nh"], True, sp["pal"], **kw))
    return GroupStream(ctx, members), oracles


@pytest.mark.parametrize("fw,fh", [(640, 360), (333, 187)])
def test_group_of_three_networks_matches_oracle(hs, ctx, fw, fh):
    specs = _specs(fw, fh)
    frames = si.tool_scene_frames(3, fh, fw, seed=40)
    grp, oracles = _build(hs, ctx, specs, fw, fh, depth=2)
    ogroup = oracle.OracleGroup([o32 for o32, _ in oracles])
    try:
        for i, f in enumerate(frames):
            print(f"[group {fw}x{fh}] frame {i}", flush=True)
            d_in, d_out = grp.upload_frame(f), grp.new_output()
            assert grp.submit(d_in, d_out, i) == hs.HS_OK
            rs = grp.wait_batch()
            assert len(rs) == 3 and all(r.frame_id == i for r in rs)
            assert len({r.t_submit_ns for r in rs}) == 1
            assert all(r.d_overlay == d_out.data_ptr() for r in rs)
            want_all = ogroup.process(f)
            picture = np.array(f, copy=True)
            for m, sp, r, (o32, o16), a in zip(grp.members, specs, rs, oracles,
                                               want_all["members"]):
                assert r.t_submit_ns <= r.t_pre_done_ns <= r.t_infer_done_ns \
                    <= r.t_post_done_ns <= r.t_overlay_done_ns <= r.t_observed_ns
                g = m.fetch(r)            # no per-member picture: the group draws one
                check_frame(g, f, a, o16.process(f), threshold=sp["thr"], alpha=sp["alpha"],
                            palette=sp["pal"], fp32_input=False, tag=f"group/{sp['name']}/f{i}")
                picture = oracle.draw_layer(picture, g["mask"], g["argmax_idx"], g["present"], o32)
            got = d_out.cpu().numpy()[:, :3 * fw].reshape(fh, fw, 3)
            assert np.array_equal(got, picture), f"frame {i}: composited overlay differs"
            # all-oracle picture: may differ only where a member's mask / argmax legitimately may
            same_inputs = all(np.array_equal(m.fetch(r)["mask"], a["mask"]) and
                              np.array_equal(m.fetch(r)["argmax_idx"], a["argmax_idx"])
                              for m, r, a in zip(grp.members, rs, want_all["members"]))
            if same_inputs:
                assert np.array_equal(got, want_all["overlay"])
    finally:
        grp.close()


@pytest.mark.parametrize("mode", ["HS_LAUNCH_EAGER", "HS_LAUNCH_GRAPH"])
def test_group_equals_members_run_alone_and_calls_are_guarded(hs, ctx, mode):
    """Two frames in flight through a group (depth 2, no wait in between; members launched kernel
    by kernel or as graphs) give bit-identical per-member outputs to the same applications run
    alone; grouped members refuse direct calls."""
    from paper_2402_04466_amd import api
    fw, fh = 640, 360
    specs = _specs(fw, fh)
    frames = si.uniform_frames(4, fh, fw, 41)
    grp, _ = _build(hs, ctx, specs, fw, fh, depth=2)
    for m in grp.members:
        hs.hs_set_launch_mode(m.app, getattr(hs, mode))
    solo, _ = _build(hs, ctx, specs, fw, fh, depth=2)
    api.hs_destroy_group(solo.group)      # the same three applications, ungrouped
    solo.group = None
    try:
        with pytest.raises(hs.HsError) as e:
            grp.members[1].submit(grp.upload_frame(frames[0]), grp.new_output(), 0)
        assert e.value.status == hs.HS_E_STATE
        with pytest.raises(hs.HsError) as e:
            api.hs_destroy_app(grp.members[0].app)
        assert e.value.status == hs.HS_E_STATE
        with pytest.raises(hs.HsError) as e:
            api.hs_create_group(ctx, [grp.members[0].app])
        assert e.value.status == hs.HS_E_STATE
        assert api.hs_poll_group(grp.group, 3) is None
        d_in = [grp.upload_frame(f) for f in frames]
        d_out = [grp.new_output() for _ in frames]
        got = []
        for k in range(0, 4, 2):
            print(f"[group overlap] frames {k}, {k + 1}", flush=True)
            assert grp.submit(d_in[k], d_out[k], k) == hs.HS_OK
            assert grp.submit(d_in[k + 1], d_out[k + 1], k + 1) == hs.HS_OK
            assert grp.submit(d_in[k], d_out[k], 99) == hs.HS_E_QUEUE_FULL
            for j in (k, k + 1):
                rs = grp.wait_batch()
                assert [r.frame_id for r in rs] == [j] * 3
                got.append([m.fetch(r) for m, r in zip(grp.members, rs)])
        for j, f in enumerate(frames):
            for mi, m in enumerate(solo.members):
                o = m.new_output()
                assert m.submit(d_in[j], o, j) == hs.HS_OK
                g = m.fetch(m.wait())
                for key in ("logits", "mask", "argmax_idx", "present", "net_input"):
                    assert np.array_equal(g[key], got[j][mi][key]), (j, mi, key)
    finally:
        grp.close()
        solo.close()


def test_mux_feeds_a_batched_application_stream_by_stream(hs, ctx):
    """Three streams of a batch-3 application hand over their frames on their own (here from
    three threads, out of order and with delays); every stream gets its own result with its own
    arrival stamp, and the outputs equal those of the same frames submitted as whole batches."""
    import threading
    import time
    from paper_2402_04466_amd import api
    from paper_2402_04466_amd.harness import AppStream
    B, T, fw, fh = 3, 4, 320, 240
    blob = si.he_normal_blob(TINY, 0)
    kw = dict(net=hs.HS_NET_TINY4, frame_w=fw, frame_h=fh, net_w=128, net_h=128, blob=blob,
              palette=PAL_A, queue_depth=T, batch=B)   # a slot per batch: buffers stay readable
    a, ref_app = AppStream(ctx, **kw), AppStream(ctx, **kw)
    mux = api.hs_create_mux(a.app, B)
    try:
        frames = [list(si.uniform_frames(T, fh, fw, 70 + j)) for j in range(B)]
        d_in = [[a.upload_frame(f) for f in frames[j]] for j in range(B)]
        d_out = [[a.new_output() for _ in range(T)] for j in range(B)]
        ref_out = [[a.new_output() for _ in range(T)] for j in range(B)]
        ref = []
        for t in range(T):
            assert ref_app.submit_batch([d_in[j][t] for j in range(B)],
                                        [ref_out[j][t] for j in range(B)], t) == hs.HS_OK
            rs = ref_app.wait_batch()
            ref.append([ref_app.fetch(rs[j], ref_out[j][t]) for j in range(B)])
        # a stream cannot run ahead of its batch
        assert api.hs_mux_submit(mux, 1, d_in[1][0].data_ptr(), d_out[1][0].data_ptr(), 100) == hs.HS_OK
        assert api.hs_mux_submit(mux, 1, d_in[1][1].data_ptr(), d_out[1][1].data_ptr(), 101) \
            == hs.HS_E_QUEUE_FULL
        assert api.hs_mux_poll(mux, 1) is None
        got = [[None] * T for _ in range(B)]
        errors = []

        def stream_thread(j):
            try:
                for t in range(T):
                    if not (j == 1 and t == 0):          # stream 1's first frame is already in
                        time.sleep(0.002 * ((j + t) % 3))
                        assert api.hs_mux_submit(mux, j, d_in[j][t].data_ptr(),
                                                 d_out[j][t].data_ptr(), 100 + t) == hs.HS_OK
                    r = api.hs_mux_wait(mux, j, 5_000_000_000)
                    assert r is not None and r.frame_id == 100 + t
                    got[j][t] = r
            except BaseException as e:      # noqa: BLE001 - reported by the main thread
                errors.append((j, repr(e)))

        print("[mux] 3 streams x 4 frames from 3 threads", flush=True)
        th = [threading.Thread(target=stream_thread, args=(j,)) for j in range(B)]
        for t_ in th:
            t_.start()
        for t_ in th:
            t_.join()
        assert not errors, errors
        for t in range(T):
            stamps = [got[j][t].t_submit_ns for j in range(B)]
            assert len(set(stamps)) == B                       # every stream its own arrival
            done = {got[j][t].t_overlay_done_ns for j in range(B)}
            assert len(done) == 1 and max(stamps) <= done.pop()  # one batch, one departure
            for j in range(B):
                g = a.fetch(got[j][t], d_out[j][t])
                for key in ("net_input", "logits", "mask", "argmax_idx", "present", "overlay"):
                    assert np.array_equal(g[key], ref[t][j][key]), (t, j, key)
        # the native driver over the same mux: one feed per stream, paced
        feeds = [{"mux": mux, "mux_stream": j, "results_per_frame": 1,
                  "frames": [[x.data_ptr()] for x in d_in[j]],
                  "outs": [[x.data_ptr()] for x in d_out[j]]} for j in range(B)]
        results, dropped, late, _ = api.hs_run_feeds(feeds, 500.0, 8)
        assert dropped == [0] * B and all(len(r) == 8 for r in results)
        for j in range(B):
            assert [r[0].frame_id for r in results[j]] == list(range(8))
            assert all(r[0].t_overlay_done_ns > r[0].t_submit_ns for r in results[j])
    finally:
        api.hs_destroy_mux(mux)
        a.close()
        ref_app.close()
