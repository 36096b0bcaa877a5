"""Stage 2 oracle: the convolutional tool-tracking network with a ConvLSTM cell.

Paper, Section III-A: an LSTM inference operator runs a pre-trained model on each
pre-processed frame; "LSTM" implies recurrent state carried from frame to frame.  The
paper does not describe the model.  The two architectures here are the synthetic
stand-ins fixed by the benchmark configurations (a 4-layer 3x3 net, and a
ResNet-18-style backbone + one ConvLSTM cell + 1x1 head); the readings are listed in
the design notes.

Every dot product is accumulated in float64 and rounded once to float32.  With
``storage="fp16"`` the weights and every stored activation tensor are additionally
rounded to half precision (nearest-even) while accumulation stays float64; this
emulates a half-precision-storage implementation and is used to separate precision
drift from kernel bugs.
"""
from __future__ import annotations

import numpy as np


def _store(x: np.ndarray, storage: str) -> np.ndarray:
    x = x.astype(np.float32)
    if storage == "fp16":
        x = x.astype(np.float16).astype(np.float32)
    return x


def conv2d(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Cross-correlation (no kernel flip), zero padding, no bias.

    y[o, Y, X] = sum_{c, dy, dx} w[o, c, dy, dx] * x[c, stride*Y + dy - pad, stride*X + dx - pad]
    x: (C, H, W); w: (O, C, k, k).  Returns float64 (O, Ho, Wo); callers round.
    The sum over c is one float64 matrix product per kernel tap.
    """
    c, h, wd = x.shape
    o, c2, k, k2 = w.shape
    assert c == c2 and k == k2
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    xp = np.zeros((c, h + 2 * pad, wd + 2 * pad), dtype=np.float64)
    xp[:, pad:pad + h, pad:pad + wd] = x
    # tap-major copy so that each per-tap (O, C) matrix is contiguous for the matmul
    w_taps = np.ascontiguousarray(w.astype(np.float64).transpose(2, 3, 0, 1))
    acc = np.zeros((o, ho * wo), dtype=np.float64)
    for dy in range(k):
        for dx in range(k):
            patch = xp[:, dy:dy + stride * (ho - 1) + 1:stride,
                       dx:dx + stride * (wo - 1) + 1:stride]
            acc += w_taps[dy, dx] @ patch.reshape(c, ho * wo)
    return acc.reshape(o, ho, wo)


def maxpool2d(x: np.ndarray, k: int = 3, stride: int = 2, pad: int = 1) -> np.ndarray:
    """Max over k x k windows; padded positions never win (treated as -inf)."""
    c, h, wd = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    xp = np.full((c, h + 2 * pad, wd + 2 * pad), -np.inf, dtype=x.dtype)
    xp[:, pad:pad + h, pad:pad + wd] = x
    out = np.full((c, ho, wo), -np.inf, dtype=x.dtype)
    for dy in range(k):
        for dx in range(k):
            out = np.maximum(out, xp[:, dy:dy + stride * (ho - 1) + 1:stride,
                                     dx:dx + stride * (wo - 1) + 1:stride])
    return out


def relu(x):
    return np.maximum(x, 0)


def sigmoid(x):
    x = np.asarray(x, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-x))


def split_blob(blob: np.ndarray, shapes):
    """Cut a flat float32 blob into [Cout][Cin][k][k] arrays, in the given order."""
    out, off = [], 0
    for (co, ci, k) in shapes:
        n = co * ci * k * k
        out.append(np.asarray(blob[off:off + n], dtype=np.float32).reshape(co, ci, k, k))
        off += n
    assert off == blob.size, "weight blob size does not match the architecture"
    return out


def basic_block(a, wa, wb, wp, stride: int, storage: str = "fp32"):
    """out = ReLU(conv3x3_b(ReLU(conv3x3_a(a))) + shortcut(a)); conv_a carries the stride;
    shortcut is the identity, or a 1x1 convolution of the same stride when ``wp`` is given."""
    t = _store(relu(conv2d(a, wa, stride, 1)), storage)
    short = a if wp is None else _store(conv2d(a, wp, stride, 0), storage)
    return _store(relu(conv2d(t, wb, 1, 1) + short), storage)


class Tiny4Net:
    """3->16 (s2) -> 32 (s2) -> 32 (s1) -> 8 (s1); 3x3, pad 1, ReLU after the first
    three layers, last layer linear (its outputs are the logits).  Stateless."""

    SHAPES = ((16, 3, 3), (32, 16, 3), (32, 32, 3), (8, 32, 3))
    STRIDES = (2, 2, 1, 1)

    def __init__(self, blob: np.ndarray, storage: str = "fp32"):
        self.storage = storage
        self.w = [_store(w, storage) for w in split_blob(blob, self.SHAPES)]

    def reset(self):
        pass

    def forward(self, x: np.ndarray) -> np.ndarray:
        a = _store(x, self.storage)
        for i, (w, s) in enumerate(zip(self.w, self.STRIDES)):
            y = conv2d(a, w, s, 1)
            if i < 3:
                a = _store(relu(y), self.storage)
            else:
                return y.astype(np.float32)


def convlstm_step(x, h, c, w, storage: str = "fp32"):
    """One ConvLSTM step without peepholes or bias.

    G = conv3x3([x ; h_prev]) with output channels ordered i, f, g, o (hid each);
    i, f, o = sigmoid, g = tanh;  c = f*c_prev + i*g;  h = o*tanh(c).
    Returns (h, c) as float32 (h optionally rounded to half precision)."""
    hid = h.shape[0]
    g_all = conv2d(np.concatenate([x, h], axis=0), w, 1, 1)
    gi = sigmoid(g_all[0 * hid:1 * hid])
    gf = sigmoid(g_all[1 * hid:2 * hid])
    gg = np.tanh(g_all[2 * hid:3 * hid])
    go = sigmoid(g_all[3 * hid:4 * hid])
    c_new = gf * c.astype(np.float64) + gi * gg
    h_new = go * np.tanh(c_new)
    return _store(h_new, storage), c_new.astype(np.float32)


class ResNet18ConvLSTMNet:
    """Stem 7x7/2 pad 3 (3->64) + ReLU, max-pool 3x3/2 pad 1, four stages of two
    BasicBlocks (widths 64/128/256/512; first block of stages 2-4 has stride 2 and a
    1x1 stride-2 projection shortcut), no normalisation layers, no bias; one ConvLSTM
    cell (512 + 256 -> 4*256, 3x3) whose state persists across frames; 1x1 head
    256 -> 8 (linear logits)."""

    HID = 256

    @staticmethod
    def shapes():
        s = [(64, 3, 7)]
        cin = 64
        for width in (64, 128, 256, 512):
            for b in range(2):
                s.append((width, cin if b == 0 else width, 3))
                s.append((width, width, 3))
                if b == 0 and cin != width:
                    s.append((width, cin, 1))
            cin = width
        s.append((4 * 256, 512 + 256, 3))
        s.append((8, 256, 1))
        return tuple(s)

    def __init__(self, blob: np.ndarray, storage: str = "fp32"):
        self.storage = storage
        ws = [_store(w, storage) for w in split_blob(blob, self.shapes())]
        it = iter(ws)
        self.stem = next(it)
        self.blocks = []
        cin = 64
        for width in (64, 128, 256, 512):
            for b in range(2):
                wa, wb = next(it), next(it)
                wp = next(it) if (b == 0 and cin != width) else None
                self.blocks.append((wa, wb, wp, 2 if wp is not None else 1))
            cin = width
        self.w_lstm = next(it)
        self.w_head = next(it)
        self.h = None
        self.c = None

    def reset(self):
        self.h = None
        self.c = None

    def features(self, x: np.ndarray) -> np.ndarray:
        st = self.storage
        a = _store(relu(conv2d(_store(x, st), self.stem, 2, 3)), st)
        a = maxpool2d(a, 3, 2, 1)
        for wa, wb, wp, stride in self.blocks:
            a = basic_block(a, wa, wb, wp, stride, st)
        return a

    def forward(self, x: np.ndarray) -> np.ndarray:
        f = self.features(x)
        if self.h is None:
            self.h = np.zeros((self.HID,) + f.shape[1:], dtype=np.float32)
            self.c = np.zeros_like(self.h)
        self.h, self.c = convlstm_step(f, self.h, self.c, self.w_lstm, self.storage)
        return conv2d(self.h, self.w_head, 1, 0).astype(np.float32)
