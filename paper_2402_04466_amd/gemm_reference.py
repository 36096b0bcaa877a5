"""Measurement aid, not part of the hot path: what the vendor GEMM library (through
``torch.matmul``, fp16 in, fp32 accumulate) reaches on plain matrix products of the same
M x N x K as the network's convolutions seen as implicit GEMMs (M = output pixels, N = output
channels, K = 9 * input channels).  A plain GEMM reads a ready-made M x K matrix, i.e. it does
not pay for gathering the nine taps, so these figures are an upper reference for a library-based
convolution and put the kernels' fraction of the MFMA peak into context.

Usage: python -m paper_2402_04466_amd.gemm_reference [--batch B]
"""
from __future__ import annotations

import argparse

import torch


def layer_shapes(batch: int):
    px = {1: 120 * 214, 2: 60 * 107, 3: 30 * 54, 4: 15 * 27}
    return [
        (f"stage 1 conv 64->64 (x{batch})", batch * px[1], 64, 576),
        (f"stage 2 conv 128->128 (x{batch})", batch * px[2], 128, 1152),
        (f"stage 3 conv 256->256 (x{batch})", batch * px[3], 256, 2304),
        (f"stage 4 conv 512->512 (x{batch})", batch * px[4], 512, 4608),
        (f"ConvLSTM gates 768->1024 (x{batch})", batch * px[4], 1024, 6912),
        ("square 8192 (library at its best)", 8192, 8192, 8192),
    ]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=12)
    args = ap.parse_args()
    print("| product | M x N x K | us | TFLOP/s |\n|---|---|---|---|")
    for name, m, n, k in layer_shapes(args.batch):
        a = torch.randn(m, k, device="cuda", dtype=torch.float16)
        b = torch.randn(k, n, device="cuda", dtype=torch.float16)
        for _ in range(5):
            a @ b
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record()
        for _ in range(reps):
            a @ b
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        print(f"| {name} | {m} x {n} x {k} | {us:.1f} | {2.0 * m * n * k / us / 1e6:.0f} |", flush=True)


if __name__ == "__main__":
    main()
