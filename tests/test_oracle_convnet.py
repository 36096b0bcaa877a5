"""Pins for the stage-2 oracle (convolutions, pooling, residual blocks, ConvLSTM):
nested-loop brute force on tiny tensors for every (k, stride, pad) used, closed forms,
algebraic invariants, and library routines (torch CPU) as independent witnesses.
The paper (Section III-A) describes no architecture and prints no outputs, so the
whole-network values are pinned only compositionally."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import (conv2d, maxpool2d, relu, basic_block, convlstm_step, Tiny4Net,
                    ResNet18ConvLSTMNet, split_blob)

CASES = [(3, 1, 1), (3, 2, 1), (1, 2, 0), (7, 2, 3), (1, 1, 0)]


def _brute_conv(x, w, stride, pad):
    c, h, wd = x.shape
    o, _, k, _ = w.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (wd + 2 * pad - k) // stride + 1
    y = np.zeros((o, ho, wo))
    for oo in range(o):
        for Y in range(ho):
            for X in range(wo):
                s = 0.0
                for cc in range(c):
                    for dy in range(k):
                        for dx in range(k):
                            iy, ix = stride * Y + dy - pad, stride * X + dx - pad
                            if 0 <= iy < h and 0 <= ix < wd:
                                s += float(w[oo, cc, dy, dx]) * float(x[cc, iy, ix])
                y[oo, Y, X] = s
    return y


@pytest.mark.parametrize("k,stride,pad", CASES)
@pytest.mark.parametrize("h,wd", [(7, 9), (8, 6)])
def test_conv_against_nested_loops(k, stride, pad, h, wd):
    rng = np.random.default_rng(k * 10 + stride)
    x = rng.standard_normal((3, h, wd)).astype(np.float32)
    w = rng.standard_normal((4, 3, k, k)).astype(np.float32)
    np.testing.assert_allclose(conv2d(x, w, stride, pad), _brute_conv(x, w, stride, pad),
                               rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("k,stride,pad", CASES)
def test_conv_against_torch_cpu(k, stride, pad):
    rng = np.random.default_rng(99 + k)
    x = rng.standard_normal((5, 21, 30)).astype(np.float32)
    w = rng.standard_normal((6, 5, k, k)).astype(np.float32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double()[None],
                                     torch.from_numpy(w).double(), stride=stride,
                                     padding=pad)[0].numpy()
    np.testing.assert_allclose(conv2d(x, w, stride, pad), ref, rtol=1e-11, atol=1e-11)


def test_delta_kernel_is_identity_and_shifted_delta_shifts():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 6, 7)).astype(np.float32)
    w = np.zeros((2, 2, 3, 3), np.float32)
    w[0, 0, 1, 1] = w[1, 1, 1, 1] = 1
    assert np.array_equal(conv2d(x, w, 1, 1), x.astype(np.float64))
    # tap (dy=0, dx=2) reads x[Y-1, X+1]: cross-correlation, not a flipped kernel
    w2 = np.zeros((1, 2, 3, 3), np.float32)
    w2[0, 1, 0, 2] = 1
    y = conv2d(x, w2, 1, 1)[0]
    assert y[3, 2] == x[1, 2, 3] and y[0, 0] == 0.0 and y[5, 6] == 0.0


def test_constant_input_interior_is_sum_of_weights():
    w = np.random.default_rng(4).standard_normal((3, 2, 3, 3)).astype(np.float32)
    y = conv2d(np.ones((2, 6, 6), np.float32), w, 1, 1)
    np.testing.assert_allclose(y[:, 1:-1, 1:-1],
                               w.astype(np.float64).sum(axis=(1, 2, 3))[:, None, None]
                               * np.ones((1, 4, 4)), rtol=1e-13)
    # corner (0,0) sees only taps dy,dx in {1,2}
    np.testing.assert_allclose(y[:, 0, 0], w.astype(np.float64)[:, :, 1:, 1:].sum(axis=(1, 2, 3)),
                               rtol=1e-13)


def test_linearity_and_stride2_is_subsampled_stride1():
    rng = np.random.default_rng(5)
    x1 = rng.standard_normal((3, 9, 11)).astype(np.float32)
    x2 = rng.standard_normal((3, 9, 11)).astype(np.float32)
    w = rng.standard_normal((4, 3, 3, 3)).astype(np.float32)
    np.testing.assert_allclose(conv2d(x1, w, 1, 1) * 2 - conv2d(x2, w, 1, 1) * 3,
                               conv2d(2 * x1.astype(np.float64) - 3 * x2.astype(np.float64), w, 1, 1),
                               atol=1e-12)
    np.testing.assert_array_equal(conv2d(x1, w, 2, 1), conv2d(x1, w, 1, 1)[:, ::2, ::2])


def test_1x1_conv_is_matrix_product():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 4, 3)).astype(np.float32)
    w = rng.standard_normal((7, 5, 1, 1)).astype(np.float32)
    ref = w[:, :, 0, 0].astype(np.float64) @ x.reshape(5, -1).astype(np.float64)
    np.testing.assert_allclose(conv2d(x, w, 1, 0).reshape(7, -1), ref, rtol=1e-13)


def test_shape_chain_of_the_1080p_configuration():
    h, w = 480, 854
    def o(n, k, s, p):
        return (n + 2 * p - k) // s + 1
    chain = [(o(h, 7, 2, 3), o(w, 7, 2, 3))]
    chain.append((o(chain[-1][0], 3, 2, 1), o(chain[-1][1], 3, 2, 1)))
    for _ in range(3):
        chain.append((o(chain[-1][0], 3, 2, 1), o(chain[-1][1], 3, 2, 1)))
    assert chain == [(240, 427), (120, 214), (60, 107), (30, 54), (15, 27)]
    # the oracle's own functions produce the same sizes on a 1-channel probe
    x = np.zeros((1, 48, 85), np.float32)
    assert conv2d(x, np.zeros((1, 1, 7, 7), np.float32), 2, 3).shape == (1, 24, 43)
    assert maxpool2d(np.zeros((1, 24, 43), np.float32)).shape == (1, 12, 22)
    assert conv2d(np.zeros((1, 12, 22), np.float32), np.zeros((1, 1, 1, 1), np.float32),
                  2, 0).shape == (1, 6, 11)


def test_maxpool_against_nested_loops_and_torch():
    rng = np.random.default_rng(7)
    x = (rng.standard_normal((3, 9, 12)) - 3.0).astype(np.float32)   # all-negative borders matter
    y = maxpool2d(x)
    for c in range(3):
        for Y in range(y.shape[1]):
            for X in range(y.shape[2]):
                vals = [x[c, iy, ix] for iy in range(2 * Y - 1, 2 * Y + 2)
                        for ix in range(2 * X - 1, 2 * X + 2)
                        if 0 <= iy < 9 and 0 <= ix < 12]
                assert y[c, Y, X] == max(vals)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x)[None], 3, 2, 1)[0].numpy()
    assert np.array_equal(y, ref)


def test_basic_block_zero_weights_is_relu_of_shortcut():
    rng = np.random.default_rng(8)
    a = rng.standard_normal((4, 6, 8)).astype(np.float32)
    z = np.zeros((4, 4, 3, 3), np.float32)
    assert np.array_equal(basic_block(a, z, z, None, 1), relu(a))
    wp = rng.standard_normal((6, 4, 1, 1)).astype(np.float32)
    za, zb = np.zeros((6, 4, 3, 3), np.float32), np.zeros((6, 6, 3, 3), np.float32)
    out = basic_block(a, za, zb, wp, 2)
    ref = relu(np.einsum("oc,chw->ohw", wp[:, :, 0, 0].astype(np.float64),
                         a[:, ::2, ::2].astype(np.float64))).astype(np.float32)
    assert np.array_equal(out, ref)


def test_basic_block_against_torch():
    rng = np.random.default_rng(9)
    a = rng.standard_normal((4, 9, 7)).astype(np.float32)
    wa = rng.standard_normal((6, 4, 3, 3)).astype(np.float32) * 0.3
    wb = rng.standard_normal((6, 6, 3, 3)).astype(np.float32) * 0.3
    wp = rng.standard_normal((6, 4, 1, 1)).astype(np.float32)
    F = torch.nn.functional
    ta = torch.from_numpy(a).double()[None]
    t = F.relu(F.conv2d(ta, torch.from_numpy(wa).double(), stride=2, padding=1))
    ref = F.relu(F.conv2d(t, torch.from_numpy(wb).double(), padding=1)
                 + F.conv2d(ta, torch.from_numpy(wp).double(), stride=2))[0].numpy()
    np.testing.assert_allclose(basic_block(a, wa, wb, wp, 2), ref, rtol=2e-6, atol=2e-6)


def test_convlstm_zero_weights_closed_form():
    hid = 3
    c0 = np.random.default_rng(10).standard_normal((hid, 4, 5)).astype(np.float32)
    h0 = np.zeros_like(c0)
    x = np.ones((2, 4, 5), np.float32)
    w = np.zeros((4 * hid, 2 + hid, 3, 3), np.float32)
    h1, c1 = convlstm_step(x, h0, c0, w)
    np.testing.assert_allclose(c1, c0 / 2, rtol=1e-7)
    np.testing.assert_allclose(h1, np.tanh(c0.astype(np.float64) / 2) / 2, rtol=1e-6)


def test_convlstm_1x1_centre_tap_is_textbook_lstm_cell():
    rng = np.random.default_rng(11)
    cx, hid = 5, 4
    w = np.zeros((4 * hid, cx + hid, 3, 3), np.float32)
    w[:, :, 1, 1] = rng.standard_normal((4 * hid, cx + hid)).astype(np.float32)
    # non-centre taps must not matter at 1x1 spatial size (they only see padding)
    w[:, :, 0, 0] = 7.0
    x = rng.standard_normal((cx, 1, 1)).astype(np.float32)
    h0 = rng.standard_normal((hid, 1, 1)).astype(np.float32)
    c0 = rng.standard_normal((hid, 1, 1)).astype(np.float32)
    h1, c1 = convlstm_step(x, h0, c0, w)
    # scalar textbook cell, gate order i, f, g, o
    sg = lambda v: 1.0 / (1.0 + math.exp(-v))
    xin = np.concatenate([x[:, 0, 0], h0[:, 0, 0]]).astype(np.float64)
    pre = w[:, :, 1, 1].astype(np.float64) @ xin
    for j in range(hid):
        i_, f_, g_, o_ = sg(pre[j]), sg(pre[hid + j]), math.tanh(pre[2 * hid + j]), sg(pre[3 * hid + j])
        cc = f_ * float(c0[j, 0, 0]) + i_ * g_
        assert abs(c1[j, 0, 0] - cc) < 1e-6
        assert abs(h1[j, 0, 0] - o_ * math.tanh(cc)) < 1e-6
    # library witness: torch.nn.LSTMCell uses the same i, f, g, o ordering
    cell = torch.nn.LSTMCell(cx, hid, bias=False).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(w[:, :cx, 1, 1]).double())
        cell.weight_hh.copy_(torch.from_numpy(w[:, cx:, 1, 1]).double())
        th, tc = cell(torch.from_numpy(x[:, 0, 0]).double()[None],
                      (torch.from_numpy(h0[:, 0, 0]).double()[None],
                       torch.from_numpy(c0[:, 0, 0]).double()[None]))
    np.testing.assert_allclose(h1[:, 0, 0], th[0].numpy(), atol=1e-6)
    np.testing.assert_allclose(c1[:, 0, 0], tc[0].numpy(), atol=1e-6)


def test_convlstm_against_torch_composition():
    rng = np.random.default_rng(12)
    cx, hid = 3, 2
    w = rng.standard_normal((4 * hid, cx + hid, 3, 3)).astype(np.float32) * 0.4
    x = rng.standard_normal((cx, 5, 6)).astype(np.float32)
    h0 = rng.standard_normal((hid, 5, 6)).astype(np.float32)
    c0 = rng.standard_normal((hid, 5, 6)).astype(np.float32)
    h1, c1 = convlstm_step(x, h0, c0, w)
    g = torch.nn.functional.conv2d(torch.from_numpy(np.concatenate([x, h0]))[None].double(),
                                   torch.from_numpy(w).double(), padding=1)[0]
    i_, f_, g_, o_ = torch.split(g, hid, dim=0)
    tc = torch.sigmoid(f_) * torch.from_numpy(c0).double() + torch.sigmoid(i_) * torch.tanh(g_)
    th = torch.sigmoid(o_) * torch.tanh(tc)
    np.testing.assert_allclose(c1, tc.numpy(), atol=1e-6)
    np.testing.assert_allclose(h1, th.numpy(), atol=1e-6)


def test_blob_layout_and_he_normal_statistics():
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    assert blob.dtype == np.float32 and blob.size == si.blob_num_floats(si.TINY4_LAYERS)
    ws = split_blob(blob, Tiny4Net.SHAPES)
    assert [w.shape for w in ws] == [(16, 3, 3, 3), (32, 16, 3, 3), (32, 32, 3, 3), (8, 32, 3, 3)]
    assert tuple((co, ci, k) for _, co, ci, k in si.RESNET18_CONVLSTM_LAYERS) == \
        ResNet18ConvLSTMNet.shapes()
    assert si.blob_num_floats(si.RESNET18_CONVLSTM_LAYERS) == 18246848
    w = ws[2]
    target = math.sqrt(2.0 / (32 * 9))
    n = w.size
    assert abs(w.std() - target) < 3 * target / math.sqrt(2 * n)
    assert abs(w.mean()) < 3 * target / math.sqrt(n)


def test_tiny4_against_torch_and_last_layer_is_linear():
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    net = Tiny4Net(blob)
    x = np.random.default_rng(13).uniform(-2, 2, (3, 128, 128)).astype(np.float32)
    y = net.forward(x)
    assert y.shape == (8, 32, 32) and y.dtype == np.float32
    assert (y < 0).any()           # no ReLU after the last layer
    F = torch.nn.functional
    t = torch.from_numpy(x).double()[None]
    for i, (w, s) in enumerate(zip(split_blob(blob, Tiny4Net.SHAPES), Tiny4Net.STRIDES)):
        t = F.conv2d(t, torch.from_numpy(w).double(), stride=s, padding=1)
        if i < 3:
            t = F.relu(t).float().double()      # the oracle stores float32 between layers
    np.testing.assert_allclose(y, t[0].numpy(), rtol=1e-5, atol=1e-5)


def _small_resnet_input(seed):
    return np.random.default_rng(seed).uniform(-2, 2, (3, 64, 96)).astype(np.float32)


def test_resnet_convlstm_state_and_reset():
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    net = ResNet18ConvLSTMNet(blob)
    x = _small_resnet_input(14)
    l1 = net.forward(x)
    assert l1.shape == (8, 2, 3) and net.h.shape == (256, 2, 3)
    l2 = net.forward(x)
    assert not np.array_equal(l1, l2)          # recurrent state carried across frames
    net.reset()
    l3 = net.forward(x)
    assert np.array_equal(l1, l3)              # reset zeroes the state


def test_resnet_features_against_torch():
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    net = ResNet18ConvLSTMNet(blob)
    x = _small_resnet_input(15)
    f = net.features(x)
    F = torch.nn.functional
    ws = [torch.from_numpy(w).double() for w in split_blob(blob, ResNet18ConvLSTMNet.shapes())]
    it = iter(ws)
    rt = lambda v: v.float().double()          # float32 storage between layers
    a = rt(F.relu(F.conv2d(torch.from_numpy(x).double()[None], next(it), stride=2, padding=3)))
    a = F.max_pool2d(a, 3, 2, 1)
    cin = 64
    for width in (64, 128, 256, 512):
        for b in range(2):
            wa, wb = next(it), next(it)
            stride = 2 if (b == 0 and cin != width) else 1
            t = rt(F.relu(F.conv2d(a, wa, stride=stride, padding=1)))
            short = a if stride == 1 else rt(F.conv2d(a, next(it), stride=2))
            a = rt(F.relu(F.conv2d(t, wb, padding=1) + short))
        cin = width
    ref = a[0].numpy()
    assert f.shape == ref.shape == (512, 2, 3)
    np.testing.assert_allclose(f, ref, rtol=1e-4, atol=1e-4 * np.abs(ref).max())


def test_fp16_storage_mode_rounds_stored_tensors_only():
    blob = si.he_normal_blob(si.TINY4_LAYERS, 0)
    x = np.random.default_rng(16).uniform(-2, 2, (3, 128, 128)).astype(np.float32)
    y32, y16 = Tiny4Net(blob).forward(x), Tiny4Net(blob, storage="fp16").forward(x)
    err = np.abs(y32 - y16).max() / np.abs(y32).max()
    assert 0 < err < 1e-2


def _torch_resnet_convlstm(blob, frames, half_storage):
    """The whole network over a frame sequence written with torch CPU routines only:
    backbone -> conv3x3([x ; h]) -> gates i, f, g, o -> (c, h) -> 1x1 head on the new h.
    float64 arithmetic; every stored tensor (and, in half-storage mode, every weight) is rounded
    to the storage type, c stays float32.  Returns per frame (logits, h, c)."""
    F = torch.nn.functional
    rt = (lambda v: v.half().double()) if half_storage else (lambda v: v.float().double())
    ws = [rt(torch.from_numpy(w)) for w in split_blob(blob, ResNet18ConvLSTMNet.shapes())]
    w_lstm, w_head = ws[-2], ws[-1]
    out, h, c = [], None, None
    for x in frames:
        it = iter(ws[:-2])
        a = rt(F.relu(F.conv2d(rt(torch.from_numpy(x))[None], next(it), stride=2, padding=3)))
        a = F.max_pool2d(a, 3, 2, 1)
        cin = 64
        for width in (64, 128, 256, 512):
            for b in range(2):
                wa, wb = next(it), next(it)
                stride = 2 if (b == 0 and cin != width) else 1
                t = rt(F.relu(F.conv2d(a, wa, stride=stride, padding=1)))
                short = a if stride == 1 else rt(F.conv2d(a, next(it), stride=2))
                a = rt(F.relu(F.conv2d(t, wb, padding=1) + short))
            cin = width
        if h is None:
            h = torch.zeros((1, 256) + tuple(a.shape[2:]), dtype=torch.float64)
            c = torch.zeros_like(h)
        g = F.conv2d(torch.cat([a, h], dim=1), w_lstm, padding=1)
        gi, gf, gg, go = torch.split(g, 256, dim=1)
        c = (torch.sigmoid(gf) * c + torch.sigmoid(gi) * torch.tanh(gg)).float().double()
        h = rt(torch.sigmoid(go) * torch.tanh(c))
        logits = F.conv2d(h, w_head).float()
        out.append((logits[0].numpy(), h[0].float().numpy(), c[0].float().numpy()))
    return out


@pytest.mark.parametrize("storage", ["fp32", "fp16"])
def test_resnet_convlstm_forward_values_against_torch_composition(storage):
    """Value pin of ResNet18ConvLSTMNet.forward, wiring included: which tensor feeds the gate
    convolution, the gate order, which of (h, c) is carried where, and that the head reads the
    NEW h.  Two frames, so that the second one runs on a non-zero carried state."""
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    frames = [_small_resnet_input(21), _small_resnet_input(22)]
    net = ResNet18ConvLSTMNet(blob, storage=storage)
    ref = _torch_resnet_convlstm(blob, frames, storage == "fp16")
    # the two float64 sums differ in order only: a stored fp16 value can flip by one step (2^-11
    # relative) where a sum lands on a rounding boundary, hence the looser bound in that mode
    tol = 1e-5 if storage == "fp32" else 2e-3
    for k, (x, (l_ref, h_ref, c_ref)) in enumerate(zip(frames, ref)):
        l = net.forward(x)
        assert l.shape == l_ref.shape == (8, 2, 3)
        for name, got, want in (("logits", l, l_ref), ("h", net.h, h_ref), ("c", net.c, c_ref)):
            err = np.abs(got - want).max() / np.abs(want).max()
            assert err <= tol, f"{storage} frame {k}: {name} off by {err:.3e}"
    # the pin can tell the mistakes it is there for: h and c are far apart, the second frame's
    # outputs depend on the carried state, and the head on c instead of h would be far off
    l2, h2, c2 = ref[1]
    assert np.abs(h2 - c2).max() > 0.05
    assert np.abs(ref[0][0] - l2).max() / np.abs(l2).max() > 1e-2
    w_head = split_blob(blob, ResNet18ConvLSTMNet.shapes())[-1]
    wrong = conv2d(c2, w_head, 1, 0)
    assert np.abs(wrong - l2).max() / np.abs(l2).max() > 10 * tol


def test_oracle_storage_modes_differ_on_the_recurrent_state_by_what_the_gpu_bound_allows():
    """The fp16-storage mode of the oracle against its fp32 mode on the recurrent state, on
    the inputs of the GPU state checks (the first four frames of the 640x360 -> 288x160 stream
    and of the 1920x1080 -> 854x480 stream).  Any half-precision-storage implementation is this far from the fp32 oracle in
    the max norm (a gate pre-activation near zero turns the rounding noise of the 20 layers in
    front of it into a visible change of h), while the rms stays small.  The GPU test's bounds
    (tests/gpu_common.py) are tied to the gap measured here: at most 1.5 times the worst one."""
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from gpu_common import TOL_STATE_MAX, TOL_STATE_RMS, rel_err, rms_rel
    import oracle
    blob = si.he_normal_blob(si.RESNET18_CONVLSTM_LAYERS, 1)
    for key, (fw, fh, nw, nh, seed, n), lo, hi in (
            ("288x160", (640, 360, 288, 160, 31, 4), 3e-2, 8e-2),
            ("854x480", (1920, 1080, 854, 480, 1, 4), 4e-2, 9e-2)):
        o32 = oracle.OracleApp("resnet18_convlstm", blob, nw, nh, True, si.DEFAULT_PALETTE)
        o16 = oracle.OracleApp("resnet18_convlstm", blob, nw, nh, True, si.DEFAULT_PALETTE,
                               storage="fp16")
        worst_max = worst_rms = worst_logits = 0.0
        stored = np.loadtxt(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                                         "config2_fp16_storage_gap.txt"), comments="#")
        for k, f in enumerate(si.tool_scene_frames(n, fh, fw, seed)):
            a, b = o32.process(f), o16.process(f)
            if key == "854x480":
                # the stored 60-frame record of this very stream (written by
                # tests/golden/make_config2_storage_gap.py from the oracle alone) starts like this
                assert stored[k, 0] == k
                assert abs(stored[k, 1] - rel_err(b["logits"], a["logits"])) <= 1e-3 * stored[k, 1]
                assert abs(stored[k, 3] - rel_err(b["h"], a["h"])) <= 1e-3 * stored[k, 3]
            worst_max = max(worst_max, rel_err(b["h"], a["h"]), rel_err(b["c"], a["c"]))
            worst_rms = max(worst_rms, rms_rel(b["h"], a["h"]), rms_rel(b["c"], a["c"]))
            worst_logits = max(worst_logits, rel_err(b["logits"], a["logits"]))
        print(f"{key}: storage-mode gap max-norm {worst_max:.3e}, rms {worst_rms:.3e}, "
              f"logits {worst_logits:.3e}")
        assert lo <= worst_max <= hi, f"{key}: max-norm gap {worst_max:.3e} outside [{lo}, {hi}]"
        assert worst_max <= TOL_STATE_MAX[key] <= 1.5 * worst_max, \
            f"{key}: TOL_STATE_MAX {TOL_STATE_MAX[key]} not within 1 .. 1.5 x {worst_max:.3e}"
        assert worst_rms <= 5e-3 and TOL_STATE_RMS >= 2 * worst_rms
        assert worst_logits <= 1e-2      # the network outputs themselves stay well inside 2e-2
