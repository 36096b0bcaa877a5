"""Writes tests/golden/input_hashes.txt: SHA-256 of the seeded synthetic inputs that the
benchmark configurations use (weight blobs and first frames), so that a change of the
generators -- or of the random-number library under them -- is noticed before any parity
figure is compared across machines.  Calls only synth_inputs/.

Usage: python tests/golden/make_input_hashes.py
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import synth_inputs as si  # noqa: E402


def entries():
    yield "weights tiny4 seed 0", si.he_normal_blob(si.TINY4_LAYERS, 0)
    yield "weights resnet18_convlstm seed 1", si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    yield "frames config1 240x320 seed 0 (8 frames)", si.uniform_frames(8, 240, 320, 0)
    for seed in (1, 2, 13):      # config 2; first stream of config 3; first stream of config 5
        frames = np.stack(list(si.tool_scene_frames(2, 1080, 1920, seed)))
        yield f"frames scene 1080x1920 seed {seed} (2 frames)", frames
    yield "palette", si.DEFAULT_PALETTE
    yield "glyphs", np.asarray(si.DEFAULT_GLYPHS, dtype=np.uint8)


def lines():
    for name, arr in entries():
        a = np.ascontiguousarray(arr)
        yield f"{hashlib.sha256(a.tobytes()).hexdigest()}  {a.dtype} {list(a.shape)}  {name}"


if __name__ == "__main__":
    with open(os.path.join(HERE, "input_hashes.txt"), "w") as fh:
        fh.write("# SHA-256 of the seeded synthetic inputs (bytes of the C-contiguous array); written by\n"
                 "# tests/golden/make_input_hashes.py from synth_inputs/ alone\n")
        for l in lines():
            fh.write(l + "\n")
            print(l)
