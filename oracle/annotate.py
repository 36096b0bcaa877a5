"""Stage 4 oracle, annotation layer: argmax markers and tool labels.

Paper, Section III-A: the visualisation operator overlays the segmented tools *and their
text labels* on the original frame.  The paper gives no geometry; the reading taken here:
for every tool channel k whose `present` flag is set, in increasing k (later tools paint
over earlier ones), on top of the mask-blended frame and fully opaque in palette[k]:

* anchor = centre of the argmax cell's footprint in the frame,
  cx = ((2*ax + 1) * Wf) // (2 * Wm), cy = ((2*ay + 1) * Hf) // (2 * Hm),
  (ay, ax) = divmod(argmax_idx[k], Wm);
* cross-hair: pixels with (|X-cx| <= arm and |Y-cy| <= half) or
  (|Y-cy| <= arm and |X-cx| <= half);
* label 'T' + digit k: two glyphs of 5 x 7 cells, each cell scale x scale pixels, the
  second glyph 6*scale pixels to the right of the first, label origin (top-left) at
  (cx + arm + 2, cy - 7*scale - 2); a pixel is painted where its glyph cell's bit is set.

Everything is clipped to the frame.  Plain nested loops over the few pixels involved.
"""
from __future__ import annotations

import numpy as np


def anchor(argmax_idx: int, wm: int, hm: int, wf: int, hf: int):
    ay, ax = divmod(int(argmax_idx), wm)
    return ((2 * ax + 1) * wf) // (2 * wm), ((2 * ay + 1) * hf) // (2 * hm)


def annotate(img: np.ndarray, argmax_idx, present, map_w: int, map_h: int, palette, glyphs,
             arm: int = 12, half: int = 1, scale: int = 2) -> np.ndarray:
    """img (Hf, Wf, 3) uint8 (already mask-blended); returns a new annotated image.
    glyphs: (9, 7) row masks, glyph 0 = 'T', glyph 1 + d = digit d; bit 4 = leftmost column."""
    out = np.array(img, dtype=np.uint8, copy=True)
    hf, wf, _ = out.shape
    pal = np.asarray(palette, dtype=np.uint8)
    gl = np.asarray(glyphs, dtype=np.int64)
    for k in range(len(present)):
        if not present[k]:
            continue
        cx, cy = anchor(argmax_idx[k], map_w, map_h, wf, hf)
        colour = pal[k]
        # cross-hair: horizontal bar, then vertical bar
        for y in range(cy - half, cy + half + 1):
            for x in range(cx - arm, cx + arm + 1):
                if 0 <= y < hf and 0 <= x < wf:
                    out[y, x] = colour
        for y in range(cy - arm, cy + arm + 1):
            for x in range(cx - half, cx + half + 1):
                if 0 <= y < hf and 0 <= x < wf:
                    out[y, x] = colour
        # label
        ox, oy = cx + arm + 2, cy - 7 * scale - 2
        for gi, g in enumerate((0, 1 + k)):
            gx0 = ox + gi * 6 * scale
            for gy in range(7):
                for gx in range(5):
                    if (gl[g, gy] >> (4 - gx)) & 1:
                        for y in range(oy + gy * scale, oy + (gy + 1) * scale):
                            for x in range(gx0 + gx * scale, gx0 + (gx + 1) * scale):
                                if 0 <= y < hf and 0 <= x < wf:
                                    out[y, x] = colour
    return out
