"""Pins of the multi-network oracle (paper Section III-B: three networks look at the same
frame in parallel, one visualisation renders the aggregated layers over the original frame).
CPU only."""
import numpy as np

import synth_inputs as si
import oracle
from oracle import OracleApp, OracleGroup, overlay, alpha_q8

PAL_A = np.array([[255, 0, 0], [0, 255, 0], [0, 0, 255], [255, 255, 0], [255, 0, 255],
                  [0, 255, 255], [255, 128, 0], [255, 255, 255]], dtype=np.uint8)
PAL_B = PAL_A[::-1].copy()


def _member(seed, net_w, net_h, pal, alpha, glyphs=None):
    return OracleApp("tiny4", si.he_normal_blob(si.TINY4_LAYERS, seed), net_w, net_h, False, pal,
                     alpha=alpha, glyphs=glyphs, marker_arm=6, marker_half=1, glyph_scale=1)


def test_group_of_one_is_the_plain_application():
    frame = si.uniform_frames(1, 96, 160, 3)[0]
    a = _member(0, 64, 64, PAL_A, 0.5, si.DEFAULT_GLYPHS)
    b = _member(0, 64, 64, PAL_A, 0.5, si.DEFAULT_GLYPHS)
    g = OracleGroup([a]).process(frame)
    r = b.process(frame)
    assert np.array_equal(g["overlay"], r["overlay"])
    assert np.array_equal(g["members"][0]["logits"], r["logits"])


def test_members_see_the_original_frame_not_each_others_drawing():
    frame = si.uniform_frames(1, 96, 160, 4)[0]
    solo = _member(1, 96, 64, PAL_B, 0.25).process(frame)
    g = OracleGroup([_member(0, 64, 64, PAL_A, 1.0), _member(1, 96, 64, PAL_B, 0.25)]).process(frame)
    assert np.array_equal(g["members"][1]["logits"], solo["logits"])
    assert np.array_equal(g["members"][1]["mask"], solo["mask"])


def test_two_layers_per_pixel_brute_force_with_different_map_sizes():
    rng = np.random.default_rng(7)
    hf, wf = 37, 53
    frame = rng.integers(0, 256, (hf, wf, 3), dtype=np.uint8)
    m1 = (rng.random((8, 5, 7)) < 0.1).astype(np.uint8)
    m2 = (rng.random((8, 4, 3)) < 0.15).astype(np.uint8)
    a1, a2 = 0.5, 0.3
    got = overlay(overlay(frame, m1, PAL_A, a1), m2, PAL_B, a2)
    q1, q2 = alpha_q8(a1), alpha_q8(a2)
    for y in range(hf):
        for x in range(wf):
            px = [int(v) for v in frame[y, x]]
            for mask, pal, q in ((m1, PAL_A, q1), (m2, PAL_B, q2)):
                _, hm, wm = mask.shape
                cell = mask[:, (y * hm) // hf, (x * wm) // wf]
                ks = [k for k in range(8) if cell[k]]
                if ks:
                    px = [(q * int(pal[ks[0]][c]) + (256 - q) * px[c] + 128) >> 8 for c in range(3)]
            assert px == [int(v) for v in got[y, x]], (x, y)


def test_group_overlay_is_the_layers_in_member_order():
    frame = si.uniform_frames(1, 96, 160, 5)[0]
    members = [_member(0, 64, 64, PAL_A, 0.5, si.DEFAULT_GLYPHS), _member(1, 96, 64, PAL_B, 0.75),
               _member(2, 32, 32, PAL_A, 0.625, si.DEFAULT_GLYPHS)]
    g = OracleGroup(members).process(frame)
    want = frame
    for m, r in zip(members, g["members"]):
        want = overlay(want, r["mask"], m.palette, m.alpha)
        if m.glyphs is not None:
            want = oracle.annotate(want, r["argmax_idx"], r["present"], r["mask"].shape[2],
                                   r["mask"].shape[1], m.palette, m.glyphs, *m.marker)
    assert np.array_equal(g["overlay"], want)
    # order matters where two layers meet: swapping two members changes the picture
    swapped = OracleGroup([members[1], members[0], members[2]]).process(frame)
    both = (g["members"][0]["mask"].any() and g["members"][1]["mask"].any())
    assert both and not np.array_equal(swapped["overlay"], g["overlay"])


def test_opaque_last_layer_wins_and_empty_layers_change_nothing():
    rng = np.random.default_rng(11)
    frame = rng.integers(0, 256, (24, 32, 3), dtype=np.uint8)
    m1 = np.zeros((8, 3, 4), np.uint8); m1[2, 1, 1] = 1
    m2 = np.zeros((8, 6, 8), np.uint8); m2[5, 2, 2] = 1       # inside m1's cell (1, 1)
    out = overlay(overlay(frame, m1, PAL_A, 0.5), m2, PAL_B, 1.0)
    ys, xs = slice(8, 12), slice(8, 12)                        # footprint of m2's cell (2, 2)
    assert (out[ys, xs] == PAL_B[5]).all()
    empty = np.zeros((8, 3, 4), np.uint8)
    assert np.array_equal(overlay(overlay(frame, empty, PAL_A, 0.5), empty, PAL_B, 0.9), frame)
