"""He-normal random weight blobs standing in for the trained tool-tracking model.

The paper's inference operator loads a trained model at run time (Section III-A); the
model is not available, so weights are drawn N(0, 2/fan_in), fan_in = Cin*kh*kw.

A blob is one flat float32 array: the layers below in order, each stored as
``[Cout][Cin][kh][kw]`` (row-major).  The tables list shapes only, so that the blob
can be sized; what each layer *does* is defined separately by each consumer.
"""
from __future__ import annotations

import numpy as np

# (name, Cout, Cin, k)
TINY4_LAYERS = (
    ("conv1", 16, 3, 3), ("conv2", 32, 16, 3), ("conv3", 32, 32, 3), ("conv4", 8, 32, 3),
)


def _resnet18_convlstm_layers():
    layers = [("stem", 64, 3, 7)]
    cin = 64
    for s, width in enumerate((64, 128, 256, 512), start=1):
        for b in range(2):
            layers.append((f"l{s}.b{b}.a", width, cin if b == 0 else width, 3))
            layers.append((f"l{s}.b{b}.b", width, width, 3))
            if b == 0 and cin != width:
                layers.append((f"l{s}.b{b}.proj", width, cin, 1))
        cin = width
    layers.append(("lstm", 4 * 256, 512 + 256, 3))
    layers.append(("head", 8, 256, 1))
    return tuple(layers)


RESNET18_CONVLSTM_LAYERS = _resnet18_convlstm_layers()


def blob_num_floats(layers) -> int:
    return sum(co * ci * k * k for _, co, ci, k in layers)


def he_normal_blob(layers, seed: int) -> np.ndarray:
    """Flat float32 blob, layers drawn in table order from ``default_rng([seed, 0])``."""
    rng = np.random.default_rng([seed, 0])
    parts = []
    for _, co, ci, k in layers:
        std = np.float32(np.sqrt(2.0 / (ci * k * k)))
        parts.append(rng.standard_normal(co * ci * k * k, dtype=np.float32) * std)
    return np.concatenate(parts)
