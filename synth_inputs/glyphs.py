"""Label glyphs for the annotation layer: input data, like the palette.

Nine glyphs of 7 rows x 5 columns, drawn by hand for this repository: 'T' followed by
the digits 0..7 (a tool label is 'T' + its channel index).  Row strings use '#' for a
set pixel; ``DEFAULT_GLYPHS`` holds them as 7 bytes per glyph, bit 4 = leftmost column.
Both the CPU oracle's tests and the GPU path's tests pass this table in; neither side
generates it.
"""
from __future__ import annotations

import numpy as np

_ROWS = {
    "T": ("#####", "..#..", "..#..", "..#..", "..#..", "..#..", "..#.."),
    "0": (".###.", "#...#", "#..##", "#.#.#", "##..#", "#...#", ".###."),
    "1": ("..#..", ".##..", "..#..", "..#..", "..#..", "..#..", ".###."),
    "2": (".###.", "#...#", "....#", "...#.", "..#..", ".#...", "#####"),
    "3": ("####.", "....#", "....#", ".###.", "....#", "....#", "####."),
    "4": ("...#.", "..##.", ".#.#.", "#..#.", "#####", "...#.", "...#."),
    "5": ("#####", "#....", "####.", "....#", "....#", "#...#", ".###."),
    "6": ("..##.", ".#...", "#....", "####.", "#...#", "#...#", ".###."),
    "7": ("#####", "....#", "...#.", "..#..", "..#..", ".#...", ".#..."),
}
GLYPH_ORDER = "T01234567"


def _pack(rows) -> list:
    return [sum(1 << (4 - x) for x in range(5) if row[x] == "#") for row in rows]


# (9, 7) uint8: glyph g, row y -> 5-bit mask, bit 4 = column 0
DEFAULT_GLYPHS = np.array([_pack(_ROWS[c]) for c in GLYPH_ORDER], dtype=np.uint8)
