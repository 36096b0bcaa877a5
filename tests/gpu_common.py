"""Shared helpers of the GPU parity tests: run frames through libhs (via the binding) and
through the CPU oracle on the same seeded inputs, and compare stage by stage."""
from __future__ import annotations

import numpy as np

import oracle
import synth_inputs as si

TOL_NET = 2e-2        # fp16 GPU vs fp32 oracle, max |diff| / max |ref| per output tensor
TOL_CELL = 2e-3       # one ConvLSTM step / head on identical fp16 inputs: fp32-accumulate vs fp64
TOL_EMU = 1.2e-2      # logits: fp16 GPU vs the oracle's fp16-storage emulation (both round every
                      # stored tensor to half precision, at decorrelated places: the distance
                      # is that of two independent roundings, not zero)
TOL_STATE_RMS = 2e-2  # end-to-end recurrent state: rms(diff) / rms(ref)
# End-to-end recurrent state, max |diff| / max |ref|, per network input size: gates near zero
# amplify the fp16 storage noise of the 20 layers before them.  Each bound is at most 1.5 times
# the distance between the oracle's own fp16-storage and fp32 modes over the first four frames
# of the same stream, which a CPU test measures (tests/test_oracle_convnet.py: 6.8e-2 and
# 8.5e-2).  It is the maximum over 10^5 values of a heavy-tailed error, so two implementations
# that round at different places differ in it by tens of per cent.
TOL_STATE_MAX = {"288x160": 0.10, "854x480": 0.125}


def rms_rel(a, ref):
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.sqrt(((a - ref) ** 2).mean()) / max(np.sqrt((ref ** 2).mean()), 1e-30))


def rel_err(a, ref):
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(a - ref).max() / max(np.abs(ref).max(), 1e-30))


def check_frame(g: dict, frame: np.ndarray, o32: dict, o16: dict | None, *, threshold, alpha,
                palette, fp32_input, mean=0.5, std=0.25, tag="", glyphs=None, marker=(12, 1, 2),
                tol_net=TOL_NET):
    """g: GPU outputs of one frame; o32 / o16: oracle outputs (fp32 storage / fp16 emulation).
    tol_net: max-norm bound on the logits against the fp32 oracle (the nominal 2e-2 unless the
    caller has a reason, stated where it passes another)."""
    # ---- stage 1: bit-exact -------------------------------------------------------------
    lut16 = oracle.normalize_lut(mean, std, fp16=True)
    want = lut16[o32["resized"]]                                   # (H, W, 3) float32 of fp16
    got = g["net_input"].astype(np.float32)
    assert np.array_equal(got[..., :3], want), f"{tag}: stage-1 fp16 tensor differs"
    assert np.all(got[..., 3] == 0), f"{tag}: stage-1 pad channel not zero"
    if fp32_input:
        lut32 = oracle.normalize_lut(mean, std, fp16=False)
        want32 = lut32[o32["resized"]].transpose(2, 0, 1)
        assert np.array_equal(g["net_input_f32"], want32), f"{tag}: stage-1 fp32 tensor differs"
    # ---- stage 2: tolerance --------------------------------------------------------------
    e32 = rel_err(g["logits"], o32["logits"])
    assert e32 <= tol_net, f"{tag}: logits vs fp32 oracle {e32:.3e} (bound {tol_net:.3e})"
    r32 = rms_rel(g["logits"], o32["logits"])
    assert r32 <= TOL_NET, f"{tag}: logits vs fp32 oracle, rms {r32:.3e}"
    print(f"[{tag}] logits vs fp32 oracle: max-norm {e32:.2e} (bound {tol_net:.2e}), rms {r32:.2e}",
          flush=True)
    if o16 is not None:
        e16 = rel_err(g["logits"], o16["logits"])
        print(f"[{tag}] logits vs fp16-storage emulation: max-norm {e16:.2e}", flush=True)
        assert e16 <= TOL_EMU, f"{tag}: logits vs fp16-emulating oracle {e16:.3e}"
    # ---- stage 3, stage-isolated: the oracle's postprocess on the GPU's own logits ---------
    p = oracle.postprocess(g["logits"], threshold)
    assert np.array_equal(g["mask"], p["mask"]), f"{tag}: mask differs"
    assert np.array_equal(g["argmax_idx"], p["argmax_idx"]), f"{tag}: argmax differs"
    assert np.array_equal(g["present"], p["present"]), f"{tag}: present differs"
    assert np.abs(g["heat"] - p["heat"]).max() <= 1e-6, f"{tag}: heat differs"
    assert np.abs(g["peak"] - p["peak"]).max() <= 1e-6, f"{tag}: peak differs"
    # end to end: mask / argmax may differ from the fp32 oracle only inside the tolerance band
    theta = float(oracle.logit_threshold(threshold))
    band = tol_net * np.abs(o32["logits"]).max()
    bad = (g["mask"] != o32["mask"]) & (np.abs(o32["logits"] - theta) > band)
    assert not bad.any(), f"{tag}: {int(bad.sum())} mask cells differ outside the band"
    ref = o32["logits"].reshape(8, -1)
    for k in range(8):
        if g["argmax_idx"][k] != o32["argmax_idx"][k]:
            gap = ref[k].max() - ref[k, g["argmax_idx"][k]]
            assert gap <= 2 * band, f"{tag}: argmax of channel {k} differs outside the band"
    # ---- stage 4, stage-isolated: the oracle's overlay with the GPU's own mask --------------
    if "overlay" in g:
        want_ov = oracle.overlay(frame, g["mask"], palette, alpha)
        if glyphs is not None:   # annotation layer from the GPU's own argmax / present
            want_ov = oracle.annotate(want_ov, g["argmax_idx"], g["present"], g["mask"].shape[2],
                                      g["mask"].shape[1], palette, glyphs, *marker)
        assert np.array_equal(g["overlay"], want_ov), f"{tag}: overlay differs"
    return e32


def make_oracles(net_name, blob, net_w, net_h, fp16_input, palette, **kw):
    o32 = oracle.OracleApp(net_name, blob, net_w, net_h, fp16_input, palette, **kw)
    o16 = oracle.OracleApp(net_name, blob, net_w, net_h, True, palette, storage="fp16", **kw)
    return o32, o16
