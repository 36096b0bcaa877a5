"""The four stages chained per frame, as one application stream (paper Section III-A:
frame -> format conversion -> recurrent inference -> postprocess -> overlay on the
original frame)."""
from __future__ import annotations

import numpy as np

from .resize import preprocess
from .convnet import Tiny4Net, ResNet18ConvLSTMNet
from .postprocess import postprocess
from .overlay import overlay
from .annotate import annotate


class OracleApp:
    def __init__(self, net: str, blob: np.ndarray, net_w: int, net_h: int, fp16_input: bool,
                 palette: np.ndarray, mean: float = 0.5, std: float = 0.25,
                 threshold: float = 0.5, alpha: float = 0.5, storage: str = "fp32",
                 glyphs=None, marker_arm: int = 12, marker_half: int = 1, glyph_scale: int = 2):
        self.net = {"tiny4": Tiny4Net, "resnet18_convlstm": ResNet18ConvLSTMNet}[net](
            blob, storage)
        self.net_w, self.net_h, self.fp16_input = net_w, net_h, fp16_input
        self.mean, self.std, self.threshold, self.alpha = mean, std, threshold, alpha
        self.palette = np.asarray(palette, dtype=np.uint8)
        # annotation layer (markers + labels) only when a glyph table is given
        self.glyphs = None if glyphs is None else np.asarray(glyphs, dtype=np.uint8)
        self.marker = (marker_arm, marker_half, glyph_scale)

    def reset(self):
        self.net.reset()

    def process(self, frame: np.ndarray) -> dict:
        resized, net_in = preprocess(frame, self.net_w, self.net_h, self.mean, self.std,
                                     self.fp16_input)
        logits = self.net.forward(net_in)
        post = postprocess(logits, self.threshold)
        out = overlay(frame, post["mask"], self.palette, self.alpha)
        if self.glyphs is not None:
            out = annotate(out, post["argmax_idx"], post["present"], logits.shape[2],
                           logits.shape[1], self.palette, self.glyphs, *self.marker)
        res = {"resized": resized, "net_input": net_in, "logits": logits, "overlay": out}
        res.update(post)
        if hasattr(self.net, "h") and self.net.h is not None:
            res["h"], res["c"] = self.net.h, self.net.c
        return res


class OracleGroup:
    """A multi-network application (paper Section III-B): every member network looks at the
    same frame, each through its own format conversion, inference and postprocess, and ONE
    visualisation draws all their layers over the original frame.  Reading taken here for
    "renders the aggregated overlaid layers": layers are drawn in member order, each member's
    mask blend followed by its annotations, every layer on top of the picture left by the
    layer before it (ordinary back-to-front compositing)."""

    def __init__(self, members):
        self.members = list(members)

    def reset(self):
        for m in self.members:
            m.reset()

    def process(self, frame: np.ndarray) -> dict:
        per_member = [m.process(frame) for m in self.members]   # each on the ORIGINAL frame
        out = np.array(frame, dtype=np.uint8, copy=True)
        for m, r in zip(self.members, per_member):
            out = draw_layer(out, r["mask"], r["argmax_idx"], r["present"], m)
        return {"members": per_member, "overlay": out}


def draw_layer(img: np.ndarray, mask, argmax_idx, present, member: OracleApp) -> np.ndarray:
    """One member's layer over img: its mask blend, then its annotations if it has any."""
    out = overlay(img, mask, member.palette, member.alpha)
    if member.glyphs is not None:
        out = annotate(out, argmax_idx, present, mask.shape[2], mask.shape[1], member.palette,
                       member.glyphs, *member.marker)
    return out
