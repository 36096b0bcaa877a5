"""CPU oracle for the per-frame tool-tracking hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct NumPy implementations of the four pipeline stages named
in the paper's Section III-A (format conversion, recurrent conv-net inference,
tool-tracking postprocess, overlay on the original frame) and of the latency
determinism metrics of Section V-A.  Integer stages are computed exactly in int64;
floating-point stages accumulate in float64 and store float32.

Nothing here is imported by the product (the HIP library and its Python binding);
only tests, the smoke check and the benchmark's CPU-baseline leg use it.  It shares
no code with the HIP path.

Pinned by tests/test_oracle_*.py (closed forms, brute force with exact rationals and
nested loops, library cross-checks).  The paper prints no numeric example of any
stage and ships no trained model, so whole-network output *values* are pinned only
compositionally (every layer type against brute force): "parity unpinned" by the paper
for the end-to-end network output.
"""
from .resize import resize_bilinear_u8, normalize_lut, preprocess
from .convnet import (conv2d, maxpool2d, relu, sigmoid, Tiny4Net, ResNet18ConvLSTMNet,
                      convlstm_step, split_blob, basic_block)
from .postprocess import postprocess, logit_threshold
from .overlay import overlay, alpha_q8
from .annotate import annotate, anchor
from .metrics import determinism_metrics, trim_count, mann_whitney_z
from .pipeline import OracleApp, OracleGroup, draw_layer

__all__ = ["resize_bilinear_u8", "normalize_lut", "preprocess", "conv2d", "maxpool2d",
           "relu", "sigmoid", "Tiny4Net", "ResNet18ConvLSTMNet", "convlstm_step",
           "split_blob", "basic_block", "postprocess", "logit_threshold", "overlay", "alpha_q8", "annotate", "anchor",
           "determinism_metrics", "trim_count", "mann_whitney_z", "OracleApp", "OracleGroup", "draw_layer"]
