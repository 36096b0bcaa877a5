"""Pins for the stage-3 (postprocess), stage-4 (overlay) and metrics oracles: closed
forms, degenerate cases, per-pixel brute force and library witnesses.  The paper gives
the metric definitions (Section V-A) and the stage order (Section III-A) but no worked
numeric example of any stage."""
import math
import os

import numpy as np
import pytest

import synth_inputs as si
import oracle
from oracle import (postprocess, logit_threshold, overlay, alpha_q8, determinism_metrics,
                    trim_count, OracleApp)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ postprocess
def test_threshold_half_is_logit_zero_and_general_value():
    assert logit_threshold(0.5) == 0.0
    assert abs(float(logit_threshold(0.75)) - math.log(3.0)) < 1e-6
    assert logit_threshold(0.25) == -logit_threshold(0.75)


def test_constant_map_argmax_is_lowest_index():
    out = postprocess(np.full((8, 5, 7), 1.5, np.float32), 0.5)
    assert np.all(out["argmax_idx"] == 0)
    assert np.all(out["present"] == 1) and np.all(out["mask"] == 1)
    np.testing.assert_allclose(out["peak"], 1 / (1 + math.exp(-1.5)), rtol=1e-6)


def test_signed_zero_tie_goes_to_lower_index():
    l = np.full((1, 2, 3), -1.0, np.float32)
    l[0, 0, 2] = -0.0
    l[0, 1, 1] = 0.0
    out = postprocess(l, 0.5)
    assert out["argmax_idx"][0] == 2
    assert out["present"][0] == 0 and out["mask"].sum() == 0     # 0 > 0 is false (strict)
    assert out["peak"][0] == 0.5


def test_single_spike_and_duplicate_spike():
    l = np.random.default_rng(0).standard_normal((8, 15, 27)).astype(np.float32)
    for k in range(8):
        l[k, (3 * k) % 15, (5 * k + 1) % 27] = 50.0
    l[5, 14, 26] = 50.0                       # later duplicate of channel 5's maximum
    out = postprocess(l, 0.5)
    want = [((3 * k) % 15) * 27 + (5 * k + 1) % 27 for k in range(8)]
    assert list(out["argmax_idx"]) == want
    assert np.array_equal(out["argmax_idx"], l.reshape(8, -1).argmax(axis=1))   # numpy: first max


def test_all_negative_map_is_empty():
    l = -np.abs(np.random.default_rng(1).standard_normal((8, 4, 4))).astype(np.float32) - 0.1
    out = postprocess(l, 0.5)
    assert out["mask"].sum() == 0 and out["present"].sum() == 0
    assert np.all(out["peak"] < 0.5)


def test_sigmoid_identities_and_mask_consistency():
    l = np.linspace(-12, 12, 8 * 6 * 6, dtype=np.float32).reshape(8, 6, 6)
    out = postprocess(l, 0.5)
    heat = out["heat"].astype(np.float64)
    assert out["heat"].dtype == np.float32
    np.testing.assert_allclose(heat + postprocess(-l, 0.5)["heat"], 1.0, atol=1e-7)
    assert np.all(np.diff(heat.ravel()) >= 0)
    assert postprocess(np.zeros((1, 1, 1), np.float32), 0.5)["heat"][0, 0, 0] == 0.5
    clear = np.abs(l) > 1e-3
    assert np.array_equal(out["mask"][clear], (heat[clear] > 0.5).astype(np.uint8))
    out3 = postprocess(l, 0.75)
    clear3 = np.abs(l - math.log(3.0)) > 1e-3
    assert np.array_equal(out3["mask"][clear3], (heat[clear3] > 0.75).astype(np.uint8))


# ------------------------------------------------------------------ overlay
PAL = si.DEFAULT_PALETTE


def _frame(h, w, seed):
    return np.random.default_rng(seed).integers(0, 256, (h, w, 3), dtype=np.uint8)


def _mask(k, h, w, seed, p=0.3):
    return (np.random.default_rng(seed).random((k, h, w)) < p).astype(np.uint8)


def test_alpha_quantisation():
    assert alpha_q8(0.0) == 0 and alpha_q8(1.0) == 256 and alpha_q8(0.5) == 128
    assert alpha_q8(-1.0) == 0 and alpha_q8(3.0) == 256
    assert alpha_q8(0.25) == 64


def test_alpha_zero_and_empty_mask_are_identity():
    f, m = _frame(24, 32, 2), _mask(8, 3, 4, 3)
    assert np.array_equal(overlay(f, m, PAL, 0.0), f)
    assert np.array_equal(overlay(f, np.zeros_like(m), PAL, 0.5), f)


def test_alpha_one_paints_palette_of_lowest_set_channel():
    f, m = _frame(24, 32, 4), _mask(8, 3, 4, 5, p=0.4)
    out = overlay(f, m, PAL, 1.0)
    for Y in range(24):
        for X in range(32):
            cell = m[:, Y * 3 // 24, X * 4 // 32]
            if cell.any():
                assert tuple(out[Y, X]) == tuple(PAL[int(np.flatnonzero(cell)[0])])
            else:
                assert tuple(out[Y, X]) == tuple(f[Y, X])


def test_brute_force_blend_ragged_cells():
    hf, wf, hm, wm = 19, 23, 4, 5          # cells of unequal pixel size
    f, m = _frame(hf, wf, 6), _mask(8, hm, wm, 7)
    out = overlay(f, m, PAL, 0.5)
    for Y in range(hf):
        for X in range(wf):
            cell = m[:, (Y * hm) // hf, (X * wm) // wf]
            if not cell.any():
                assert tuple(out[Y, X]) == tuple(f[Y, X])
                continue
            k = int(np.flatnonzero(cell)[0])
            for c in range(3):
                assert out[Y, X, c] == (128 * int(PAL[k, c]) + 128 * int(f[Y, X, c]) + 128) >> 8


def test_changed_pixel_count_equals_cell_areas():
    hf, wf, hm, wm = 40, 50, 3, 7
    f = np.zeros((hf, wf, 3), np.uint8)          # black, so every blended pixel changes
    m = _mask(8, hm, wm, 8)
    m[:, :, :] &= 1
    out = overlay(f, m, PAL, 0.5)
    xs = [sum(1 for X in range(wf) if X * wm // wf == j) for j in range(wm)]
    ys = [sum(1 for Y in range(hf) if Y * hm // hf == i) for i in range(hm)]
    assert sum(xs) == wf and sum(ys) == hf
    want = sum(ys[i] * xs[j] for i in range(hm) for j in range(wm) if m[:, i, j].any())
    assert int((out != f).any(axis=2).sum()) == want


def test_frame_equal_to_colour_is_fixed_point_for_any_alpha():
    m = np.zeros((8, 2, 2), np.uint8)
    m[6] = 1
    f = np.tile(PAL[6][None, None, :], (10, 10, 1))
    for a in (0.1, 0.37, 0.5, 0.9, 1.0):
        assert np.array_equal(overlay(f, m, PAL, a), f)


# ------------------------------------------------------------------ metrics
def test_metrics_golden_1_to_101():
    want = {}
    with open(os.path.join(GOLDEN, "latency_1_to_101.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                want[k] = float(v)
    m = determinism_metrics(np.arange(1, 102)[::-1], trim=False)   # order must not matter
    assert m["n"] == 101 and m["p50"] == want["p50"] and m["max"] == want["max"]
    assert m["mean"] == want["mean"] and m["tail"] == want["tail"]
    assert m["flatness"] == want["flatness"]
    assert abs(m["std"] - want["std"]) < 1e-12


def test_metrics_against_numpy_estimators():
    x = np.random.default_rng(9).gamma(2.0, 3.0, 977)
    m = determinism_metrics(x, trim=False)
    assert abs(m["flatness"] - (np.percentile(x, 90) - np.percentile(x, 10))) < 1e-9
    assert abs(m["tail"] - (x.max() - np.percentile(x, 95))) < 1e-9
    assert abs(m["p99"] - np.percentile(x, 99)) < 1e-9
    assert abs(m["std"] - np.std(x)) < 1e-9 and abs(m["mean"] - np.mean(x)) < 1e-9


def test_trimming_rule():
    assert trim_count(1000) == 10 and trim_count(60) == 10 and trim_count(8) == 1
    x = np.concatenate([[1000.0] * 10, np.arange(40.0), [2000.0] * 10])
    m = determinism_metrics(x)
    assert m["n"] == 40 and m["max"] == 39.0
    assert determinism_metrics([5.0, 1.0, 2.0, 3.0, 4.0, 1.5, 2.5, 9.0])["n"] == 6


# ------------------------------------------------------------------ pipeline
def test_pipeline_stage_order_and_shapes():
    frames = si.uniform_frames(2, 240, 320, 0)
    app = OracleApp("tiny4", si.he_normal_blob(si.TINY4_LAYERS, 0), 128, 128, False, PAL)
    r = app.process(frames[0])
    assert r["net_input"].shape == (3, 128, 128) and r["logits"].shape == (8, 32, 32)
    assert r["overlay"].shape == frames[0].shape and r["overlay"].dtype == np.uint8
    # the overlay is drawn on the ORIGINAL frame: unmasked cells keep the input pixels
    cell_y = (np.arange(240) * 32) // 240
    cell_x = (np.arange(320) * 32) // 320
    untouched = ~r["mask"].any(axis=0)[cell_y][:, cell_x]
    assert np.array_equal(r["overlay"][untouched], frames[0][untouched])
    assert (r["overlay"][~untouched] != frames[0][~untouched]).any()


# ---- annotation layer (markers + labels): Section III-A, "segmented tools and their text labels" --
def _annotate_witness(img, argmax_idx, present, wm, hm, palette, glyphs, arm, half, scale, pad=64):
    """Independent construction: whole-array masks (|dx|, |dy| tests by broadcasting, glyphs by
    np.kron) on a canvas padded by `pad` on every side, cropped at the end (clipping for free)."""
    hf, wf, _ = img.shape
    canvas = np.zeros((hf + 2 * pad, wf + 2 * pad, 3), np.uint8)
    canvas[pad:pad + hf, pad:pad + wf] = img
    ys = np.arange(-pad, hf + pad)[:, None]
    xs = np.arange(-pad, wf + pad)[None, :]
    for k in range(8):
        if not present[k]:
            continue
        ay, ax = divmod(int(argmax_idx[k]), wm)
        cx = int(np.floor((ax + 0.5) * wf / wm + 1e-9))
        cy = int(np.floor((ay + 0.5) * hf / hm + 1e-9))
        dx, dy = np.abs(xs - cx), np.abs(ys - cy)
        cross = ((dx <= arm) & (dy <= half)) | ((dy <= arm) & (dx <= half))
        canvas[cross] = palette[k]
        for gi, g in enumerate((0, 1 + k)):
            bits = np.array([[(int(glyphs[g, r]) >> (4 - c)) & 1 for c in range(5)] for r in range(7)])
            big = np.kron(bits, np.ones((scale, scale), dtype=int)).astype(bool)
            oy = cy - 7 * scale - 2 + pad
            ox = cx + arm + 2 + gi * 6 * scale + pad
            region = canvas[oy:oy + 7 * scale, ox:ox + 5 * scale]
            region[big] = palette[k]
    return canvas[pad:pad + hf, pad:pad + wf]


def test_annotate_nothing_present_is_identity():
    rng = np.random.default_rng(0)
    img = rng.integers(0, 256, (40, 60, 3), dtype=np.uint8)
    out = oracle.annotate(img, [3] * 8, [0] * 8, 6, 4, si.DEFAULT_PALETTE, si.DEFAULT_GLYPHS)
    assert np.array_equal(out, img)


def test_annotate_anchor_closed_form_and_cross_pixel_count():
    # frame an integer multiple s of the map: anchor = cell origin + s // 2
    assert oracle.anchor(2 * 27 + 5, 27, 15, 27 * 70, 15 * 70) == (5 * 70 + 35, 2 * 70 + 35)
    assert oracle.anchor(0, 27, 15, 1920, 1080) == (1920 // 54, 1080 // 30)
    img = np.zeros((200, 200, 3), np.uint8)
    no_glyphs = np.zeros((9, 7), np.uint8)
    for arm, half in ((12, 1), (5, 0), (20, 3)):
        out = oracle.annotate(img, [55] + [0] * 7, [1] + [0] * 7, 10, 10, si.DEFAULT_PALETTE,
                              no_glyphs, arm, half, 2)
        painted = int((out != 0).any(axis=2).sum())
        assert painted == 2 * (2 * arm + 1) * (2 * half + 1) - (2 * half + 1) ** 2
        assert (out[(out != 0).any(axis=2)] == si.DEFAULT_PALETTE[0]).all()


@pytest.mark.parametrize("wf,hf,wm,hm,scale,arm,half", [
    (320, 240, 32, 32, 2, 12, 1),      # config-1 geometry
    (1920, 1080, 27, 15, 2, 12, 1),    # config-2 geometry
    (97, 61, 5, 3, 3, 7, 2),           # odd sizes, everything near the borders
])
def test_annotate_matches_whole_array_witness_with_clipping_and_order(wf, hf, wm, hm, scale, arm,
                                                                      half):
    rng = np.random.default_rng(wf)
    img = rng.integers(0, 256, (hf, wf, 3), dtype=np.uint8)
    n = wm * hm
    # corners (clipping on every side), two tools on the same cell (order), random others
    argmax_idx = [0, wm - 1, n - wm, n - 1, n // 2, n // 2, int(rng.integers(n)), int(rng.integers(n))]
    present = [1, 1, 1, 1, 1, 1, 0, 1]
    out = oracle.annotate(img, argmax_idx, present, wm, hm, si.DEFAULT_PALETTE, si.DEFAULT_GLYPHS,
                          arm, half, scale)
    want = _annotate_witness(img, argmax_idx, present, wm, hm, si.DEFAULT_PALETTE,
                             si.DEFAULT_GLYPHS, arm, half, scale)
    assert np.array_equal(out, want)
    cx, cy = oracle.anchor(n // 2, wm, hm, wf, hf)
    assert tuple(out[cy, cx]) == tuple(si.DEFAULT_PALETTE[5])     # tool 5 painted over tool 4
    assert np.array_equal(img, np.asarray(img))                   # input untouched


def test_glyph_table_shape_and_t_glyph():
    g = si.DEFAULT_GLYPHS
    assert g.shape == (9, 7) and g.dtype == np.uint8 and int(g.max()) < 32
    assert g[0, 0] == 0b11111 and all(int(v) == 0b00100 for v in g[0, 1:])   # 'T'
    assert len({tuple(r) for r in g}) == 9                                    # all glyphs differ


# ---- Mann-Whitney U (appendix "Additional Evaluation": |Z| > 1.96, two-tailed, 0.05) -------------
def test_mann_whitney_closed_forms():
    # complete separation: U = n*m (or 0); symmetric samples: U = n*m/2, z = 0
    r = oracle.mann_whitney_z([5, 6, 7, 8], [1, 2, 3])
    assert r["u"] == 12.0
    assert oracle.mann_whitney_z([1, 2, 3], [5, 6, 7, 8])["u"] == 0.0
    r = oracle.mann_whitney_z([1, 4], [2, 3])
    assert r["u"] == 2.0 and r["z"] == 0.0 and not r["significant"]
    # all values equal: every pair is a tie, no evidence either way
    r = oracle.mann_whitney_z([3, 3, 3], [3, 3])
    assert r["u"] == 3.0 and r["z"] == 0.0
    # hand-computed, no ties: a = {1, 3, 5}, b = {2, 4}: pairs a>b: (3,2), (5,2), (5,4) -> U = 3,
    # mu = 3, z = 0;  a = {4, 5, 6}, b = {1, 2, 3}: U = 9, mu = 4.5, var = 9*7/12 = 5.25
    assert oracle.mann_whitney_z([1, 3, 5], [2, 4])["u"] == 3.0
    r = oracle.mann_whitney_z([4, 5, 6], [1, 2, 3])
    assert r["u"] == 9.0 and abs(r["z"] - (9 - 4.5 - 0.5) / math.sqrt(5.25)) < 1e-12
    # antisymmetry
    a, b = [0.31, 0.35, 0.33, 0.40, 0.31], [0.30, 0.31, 0.29, 0.36]
    assert abs(oracle.mann_whitney_z(a, b)["z"] + oracle.mann_whitney_z(b, a)["z"]) < 1e-12
    assert oracle.mann_whitney_z(a, b)["u"] + oracle.mann_whitney_z(b, a)["u"] == len(a) * len(b)


def test_mann_whitney_against_scipy_asymptotic():
    from scipy import stats
    rng = np.random.default_rng(5)
    for n, m, shift, quant in ((40, 55, 0.0, None), (120, 80, 0.3, None), (200, 200, 0.1, 0.05),
                               (15, 9, 1.0, 0.5)):
        a = rng.normal(1.0 + shift, 0.2, n)
        b = rng.normal(1.0, 0.3, m)
        if quant:                                  # quantised latencies: many ties
            a, b = np.round(a / quant) * quant, np.round(b / quant) * quant
        got = oracle.mann_whitney_z(a, b)
        ref = stats.mannwhitneyu(a, b, alternative="two-sided", method="asymptotic",
                                 use_continuity=True)
        assert abs(got["u"] - ref.statistic) < 1e-9
        p = 2.0 * stats.norm.sf(abs(got["z"]))
        assert abs(p - ref.pvalue) <= 1e-12 + 1e-9 * ref.pvalue
        assert got["significant"] == (ref.pvalue < 2.0 * stats.norm.sf(1.96))
