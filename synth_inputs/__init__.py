"""Seeded synthetic inputs (frames and weight blobs) for the tool-tracking hot path.

This package only draws random numbers and lays them out (plus two fixed input tables: the
overlay palette and the label glyph bitmaps); it contains none of the
pipeline's arithmetic (no resize, convolution, thresholding or blending).  It is the
one module that both the CPU oracle's tests and the GPU path's tests may import.
"""
from .frames import uniform_frames, tool_scene_frames, DEFAULT_PALETTE
from .glyphs import DEFAULT_GLYPHS, GLYPH_ORDER
from .weights import (TINY4_LAYERS, RESNET18_CONVLSTM_LAYERS, he_normal_blob,
                      blob_num_floats)

__all__ = ["uniform_frames", "tool_scene_frames", "DEFAULT_PALETTE", "DEFAULT_GLYPHS",
           "GLYPH_ORDER", "TINY4_LAYERS",
           "RESNET18_CONVLSTM_LAYERS", "he_normal_blob", "blob_num_floats"]
