"""Writes tests/golden/config2_fp16_storage_gap.txt: for each of the 60 frames of the config-2
stream (1920x1080 seed-1 scene -> 854x480, ResNet-18-style + ConvLSTM, state carried 0 -> 59)
the distance between the oracle's fp16-storage mode and its fp32 mode, on the logits and on the
recurrent state.  It is the error any implementation that stores activations in half precision
shows against the fp32 oracle; the 60-frame GPU parity test takes its envelope as the bound
where it exceeds the nominal 2e-2.  Calls only oracle/ and synth_inputs/ (about four minutes
of CPU).

Usage: python tests/golden/make_config2_storage_gap.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
import synth_inputs as si  # noqa: E402


def max_rel(a, ref):
    return float(np.abs(a.astype(np.float64) - ref).max() / np.abs(ref).max())


def rms_rel(a, ref):
    a, ref = a.astype(np.float64), ref.astype(np.float64)
    return float(np.sqrt(((a - ref) ** 2).mean()) / np.sqrt((ref ** 2).mean()))


def lines(n_frames=60):
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    o32 = oracle.OracleApp("resnet18_convlstm", blob, 854, 480, True, si.DEFAULT_PALETTE)
    o16 = oracle.OracleApp("resnet18_convlstm", blob, 854, 480, True, si.DEFAULT_PALETTE,
                           storage="fp16")
    yield "# frame  logits_max logits_rms  h_max h_rms  c_max c_rms   (fp16-storage vs fp32 oracle)"
    for k, f in enumerate(si.tool_scene_frames(n_frames, 1080, 1920, 1)):
        a, b = o32.process(f), o16.process(f)
        vals = []
        for key in ("logits", "h", "c"):
            vals += [max_rel(b[key], a[key]), rms_rel(b[key], a[key])]
        yield "%d " % k + " ".join("%.4e" % v for v in vals)


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config2_fp16_storage_gap.txt")
    with open(out + ".tmp", "w") as fh:
        for line in lines():
            print(line, flush=True)
            fh.write(line + "\n")
    os.replace(out + ".tmp", out)
