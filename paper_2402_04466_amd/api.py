"""ctypes binding of libhs (see include/hs.h for the contract of every call).

Each function has the name of the C entry point it wraps and only marshals arguments:
device pointers are passed as integers (e.g. ``tensor.data_ptr()``), host arrays as NumPy
arrays.  Failing calls raise :class:`HsError`, except the two "try again" statuses
(HS_E_NOT_READY, HS_E_QUEUE_FULL), which are returned to the caller.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

__all__ = [
    "HS_OK", "HS_E_INVAL", "HS_E_NOMEM", "HS_E_OVERSUBSCRIBED", "HS_E_QUEUE_FULL",
    "HS_E_NOT_READY", "HS_E_DEVICE", "HS_E_STATE", "HS_NET_TINY4", "HS_NET_RESNET18_CONVLSTM",
    "HS_NUM_TOOLS", "HS_MAX_CU_WORDS", "HsError", "hs_app_desc", "hs_result",
    "hs_latency_metrics", "hs_kernel_time", "lib_path", "load", "hs_init", "hs_shutdown",
    "hs_device_cus", "hs_query_workspace", "hs_create_app", "hs_destroy_app", "hs_reset_state",
    "hs_get_state", "hs_get_features", "hs_set_partition", "hs_admission_check", "hs_submit_frame",
    "hs_submit_frame_static_scratch",
    "hs_poll_result", "hs_wait_result", "hs_submit_batch", "hs_submit_batch_after", "hs_poll_batch",
    "hs_wait_batch",
    "hs_create_group", "hs_destroy_group", "hs_submit_group", "hs_poll_group", "hs_wait_group",
    "HS_MAX_GROUP", "hs_feed", "hs_run_feeds", "hs_create_mux", "hs_destroy_mux", "hs_mux_submit",
    "hs_mux_poll", "hs_mux_wait", "hs_latency_metrics_compute", "hs_mann_whitney_u", "hs_set_cpu_affinity", "hs_set_kernel_timing", "hs_set_launch_mode", "HS_LAUNCH_GRAPH", "HS_LAUNCH_EAGER",
    "hs_get_kernel_times", "hs_device_copy", "hs_partition_copy", "hs_last_error", "hs_version", "make_desc", "cu_mask_words",
]

HS_OK, HS_E_INVAL, HS_E_NOMEM, HS_E_OVERSUBSCRIBED = 0, -1, -2, -3
HS_E_QUEUE_FULL, HS_E_NOT_READY, HS_E_DEVICE, HS_E_STATE = -4, -5, -6, -7
HS_NET_TINY4, HS_NET_RESNET18_CONVLSTM = 1, 2
HS_NUM_TOOLS, HS_MAX_CU_WORDS = 8, 8
HS_LAUNCH_GRAPH, HS_LAUNCH_EAGER = 0, 1
HS_MAX_GROUP = 4

_STATUS_NAME = {0: "HS_OK", -1: "HS_E_INVAL", -2: "HS_E_NOMEM", -3: "HS_E_OVERSUBSCRIBED",
                -4: "HS_E_QUEUE_FULL", -5: "HS_E_NOT_READY", -6: "HS_E_DEVICE", -7: "HS_E_STATE"}


class HsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAME.get(status, status)}: {message}")
        self.status = status


class hs_app_desc(C.Structure):
    _fields_ = [
        ("frame_w", C.c_int), ("frame_h", C.c_int), ("frame_pitch", C.c_size_t),
        ("net_w", C.c_int), ("net_h", C.c_int), ("net_fp32_input", C.c_int),
        ("mean", C.c_float), ("std", C.c_float), ("threshold", C.c_float), ("alpha", C.c_float),
        ("net", C.c_int), ("weights", C.c_void_p), ("weight_floats", C.c_size_t),
        ("palette", (C.c_uint8 * 3) * HS_NUM_TOOLS), ("queue_depth", C.c_int), ("batch", C.c_int),
        ("annotate", C.c_int), ("marker_arm", C.c_int), ("marker_half", C.c_int),
        ("glyph_scale", C.c_int), ("glyphs", (C.c_uint8 * 7) * 9),
        ("d_workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


class hs_result(C.Structure):
    _fields_ = [
        ("frame_id", C.c_uint64),
        ("t_submit_ns", C.c_uint64), ("t_enqueued_ns", C.c_uint64), ("t_pre_done_ns", C.c_uint64),
        ("t_infer_done_ns", C.c_uint64), ("t_post_done_ns", C.c_uint64),
        ("t_overlay_done_ns", C.c_uint64), ("t_observed_ns", C.c_uint64),
        ("argmax_idx", C.c_int32 * HS_NUM_TOOLS), ("present", C.c_uint8 * HS_NUM_TOOLS),
        ("peak", C.c_float * HS_NUM_TOOLS),
        ("map_w", C.c_int), ("map_h", C.c_int), ("net_input_pitch_bytes", C.c_size_t),
        ("d_overlay", C.c_void_p), ("d_mask", C.c_void_p), ("d_heat", C.c_void_p),
        ("d_logits", C.c_void_p), ("d_net_input", C.c_void_p), ("d_net_input_f32", C.c_void_p),
    ]


class hs_latency_metrics(C.Structure):
    _fields_ = [("n", C.c_uint64), ("mean", C.c_double), ("max", C.c_double), ("std", C.c_double),
                ("p50", C.c_double), ("p99", C.c_double), ("tail", C.c_double),
                ("flatness", C.c_double)]


class hs_mwu(C.Structure):
    _fields_ = [("u", C.c_double), ("z", C.c_double), ("significant", C.c_int)]


class hs_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_uint64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


_lib = None


class hs_feed(C.Structure):
    _fields_ = [("app", C.c_void_p), ("group", C.c_void_p), ("mux", C.c_void_p),
                ("mux_stream", C.c_int), ("d_frames", C.c_void_p),
                ("d_outs", C.c_void_p), ("n_frames", C.c_int), ("n_outs", C.c_int),
                ("batch", C.c_int), ("results_per_frame", C.c_int), ("cpu", C.c_int)]


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhs.so")


def load() -> C.CDLL:
    """Load libhs.so (once).  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        raise HsError(HS_E_DEVICE, f"{path} is missing: build it with "
                                   "`python -m paper_2402_04466_amd.build`")
    # PyTorch (the caller's source of device memory) ships its own copy of the HIP runtime.  It
    # has to be loaded first: if libhs binds to another copy before it, the process ends up
    # with two runtimes and torch finds no GPU.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    P = C.POINTER
    sig = {
        "hs_init": (C.c_int, [C.c_int, P(C.c_void_p)]),
        "hs_shutdown": (C.c_int, [C.c_void_p]),
        "hs_device_cus": (C.c_int, [C.c_void_p, P(C.c_int)]),
        "hs_query_workspace": (C.c_int, [P(hs_app_desc), P(C.c_size_t)]),
        "hs_create_app": (C.c_int, [C.c_void_p, P(hs_app_desc), P(C.c_void_p)]),
        "hs_destroy_app": (C.c_int, [C.c_void_p]),
        "hs_reset_state": (C.c_int, [C.c_void_p]),
        "hs_get_state": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]),
        "hs_get_features": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p]),
        "hs_submit_batch": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64]),
        "hs_submit_batch_after": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                            C.c_void_p]),
        "hs_poll_batch": (C.c_int, [C.c_void_p, P(hs_result)]),
        "hs_wait_batch": (C.c_int, [C.c_void_p, P(hs_result), C.c_uint64]),
        "hs_set_partition": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]),
        "hs_admission_check": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]),
        "hs_submit_frame": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64]),
        "hs_submit_frame_static_scratch": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_uint64]),
        "hs_poll_result": (C.c_int, [C.c_void_p, P(hs_result)]),
        "hs_wait_result": (C.c_int, [C.c_void_p, P(hs_result), C.c_uint64]),
        "hs_create_group": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int, P(C.c_void_p)]),
        "hs_destroy_group": (C.c_int, [C.c_void_p]),
        "hs_submit_group": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64]),
        "hs_poll_group": (C.c_int, [C.c_void_p, P(hs_result)]),
        "hs_wait_group": (C.c_int, [C.c_void_p, P(hs_result), C.c_uint64]),
        "hs_create_mux": (C.c_int, [C.c_void_p, C.c_int, P(C.c_void_p)]),
        "hs_destroy_mux": (C.c_int, [C.c_void_p]),
        "hs_mux_submit": (C.c_int, [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_uint64]),
        "hs_mux_poll": (C.c_int, [C.c_void_p, C.c_int, P(hs_result)]),
        "hs_mux_wait": (C.c_int, [C.c_void_p, C.c_int, P(hs_result), C.c_uint64]),
        "hs_run_feeds": (C.c_int, [P(hs_feed), C.c_int, C.c_double, C.c_int, C.c_void_p,
                                   P(C.c_int), C.c_void_p, P(C.c_double)]),
        "hs_latency_metrics_compute": (C.c_int, [C.c_void_p, C.c_size_t, C.c_int,
                                                 P(hs_latency_metrics)]),
        "hs_mann_whitney_u": (C.c_int, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, P(hs_mwu)]),
        "hs_set_cpu_affinity": (C.c_int, [C.c_void_p, C.c_int]),
        "hs_set_kernel_timing": (C.c_int, [C.c_void_p, C.c_int]),
        "hs_set_launch_mode": (C.c_int, [C.c_void_p, C.c_int]),
        "hs_get_kernel_times": (C.c_int, [C.c_void_p, P(hs_kernel_time), C.c_int, P(C.c_int)]),
        "hs_device_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]),
        "hs_partition_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int,
                                        P(C.c_double)]),
        "hs_last_error": (C.c_char_p, []),
        "hs_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def hs_last_error() -> str:
    return load().hs_last_error().decode()


def hs_version() -> str:
    return load().hs_version().decode()


def _check(status: int, soft=()) -> int:
    if status != HS_OK and status not in soft:
        raise HsError(status, hs_last_error())
    return status


def make_desc(*, frame_w, frame_h, net_w, net_h, net, weights, palette, d_workspace=0,
              workspace_bytes=0, frame_pitch=None, net_fp32_input=0, mean=0.5, std=0.25,
              threshold=0.5, alpha=0.5, queue_depth=2, batch=1, glyphs=None, marker_arm=12,
              marker_half=1, glyph_scale=2) -> hs_app_desc:
    """Fill an hs_app_desc.  ``weights`` is a contiguous float32 NumPy array (kept alive by
    the returned object); ``palette`` an (8, 3) uint8 array; ``glyphs`` a (9, 7) uint8 table of
    row masks, which switches the annotation layer (markers + labels) on."""
    d = hs_app_desc()
    d.frame_w, d.frame_h = int(frame_w), int(frame_h)
    d.frame_pitch = int(frame_pitch if frame_pitch is not None else 3 * frame_w)
    d.net_w, d.net_h, d.net_fp32_input = int(net_w), int(net_h), int(net_fp32_input)
    d.mean, d.std, d.threshold, d.alpha = mean, std, threshold, alpha
    d.net = int(net)
    w = np.ascontiguousarray(weights, dtype=np.float32)
    d._keepalive = w
    d.weights = w.ctypes.data
    d.weight_floats = w.size
    pal = np.asarray(palette, dtype=np.uint8).reshape(HS_NUM_TOOLS, 3)
    for k in range(HS_NUM_TOOLS):
        for c in range(3):
            d.palette[k][c] = int(pal[k, c])
    d.queue_depth = int(queue_depth)
    d.batch = int(batch)
    d.annotate = 0 if glyphs is None else 1
    d.marker_arm, d.marker_half, d.glyph_scale = int(marker_arm), int(marker_half), int(glyph_scale)
    if glyphs is not None:
        gl = np.asarray(glyphs, dtype=np.uint8).reshape(9, 7)
        for g in range(9):
            for r in range(7):
                d.glyphs[g][r] = int(gl[g, r])
    d.d_workspace = int(d_workspace)
    d.workspace_bytes = int(workspace_bytes)
    return d


def cu_mask_words(cus, n_words: int = HS_MAX_CU_WORDS) -> np.ndarray:
    """Bit set (uint32 words) naming the given CU indices."""
    m = np.zeros(n_words, dtype=np.uint32)
    for cu in cus:
        m[cu // 32] |= np.uint32(1 << (cu % 32))
    return m


def hs_init(device: int = 0) -> int:
    ctx = C.c_void_p()
    _check(load().hs_init(device, C.byref(ctx)))
    return ctx.value


def hs_shutdown(ctx: int) -> None:
    _check(load().hs_shutdown(ctx))


def hs_device_cus(ctx: int) -> int:
    n = C.c_int()
    _check(load().hs_device_cus(ctx, C.byref(n)))
    return n.value


def hs_query_workspace(desc: hs_app_desc) -> int:
    n = C.c_size_t()
    _check(load().hs_query_workspace(C.byref(desc), C.byref(n)))
    return n.value


def hs_create_app(ctx: int, desc: hs_app_desc) -> int:
    app = C.c_void_p()
    _check(load().hs_create_app(ctx, C.byref(desc), C.byref(app)))
    return app.value


def hs_destroy_app(app: int) -> None:
    _check(load().hs_destroy_app(app))


def hs_reset_state(app: int) -> None:
    _check(load().hs_reset_state(app))


def hs_get_state(app: int, map_h: int, map_w: int, hid: int = 256, stream: int = 0):
    """Returns (h, c) of one stream as float32 arrays of shape (hid, map_h, map_w)."""
    h = np.empty((hid, map_h, map_w), dtype=np.float32)
    c = np.empty((hid, map_h, map_w), dtype=np.float32)
    _check(load().hs_get_state(app, stream, h.ctypes.data, c.ctypes.data))
    return h, c


def hs_get_features(app: int, map_h: int, map_w: int, ch: int = 512, stream: int = 0) -> np.ndarray:
    """Returns the ConvLSTM cell's input of the last frame, float32 (ch, map_h, map_w)."""
    x = np.empty((ch, map_h, map_w), dtype=np.float32)
    _check(load().hs_get_features(app, stream, x.ctypes.data))
    return x


def hs_set_partition(app: int, cu_mask_infer, cu_mask_overlay) -> None:
    """Masks: uint32 NumPy arrays of equal length (<= 8 words), or both None to release."""
    if cu_mask_infer is None and cu_mask_overlay is None:
        _check(load().hs_set_partition(app, None, None, 0))
        return
    a = np.ascontiguousarray(cu_mask_infer, dtype=np.uint32)
    b = np.ascontiguousarray(cu_mask_overlay, dtype=np.uint32)
    if a.size != b.size:
        raise ValueError("masks must have the same number of words")
    _check(load().hs_set_partition(app, a.ctypes.data, b.ctypes.data, a.size))


def hs_admission_check(claimed_by_others, req_infer, req_overlay, device_cus: int) -> int:
    """Returns the status (HS_OK, HS_E_OVERSUBSCRIBED or HS_E_INVAL); never raises."""
    a = np.ascontiguousarray(req_infer, dtype=np.uint32)
    b = np.ascontiguousarray(req_overlay, dtype=np.uint32)
    cl = None if claimed_by_others is None else np.ascontiguousarray(claimed_by_others,
                                                                     dtype=np.uint32)
    return load().hs_admission_check(None if cl is None else cl.ctypes.data, a.ctypes.data,
                                     b.ctypes.data, a.size, device_cus)


def hs_submit_frame(app: int, d_frame: int, d_overlay_out: int, frame_id: int) -> int:
    """Returns HS_OK or HS_E_QUEUE_FULL; raises on any other status."""
    return _check(load().hs_submit_frame(app, d_frame, d_overlay_out, frame_id),
                  soft=(HS_E_QUEUE_FULL,))


def hs_submit_frame_static_scratch(app: int, d_frame: int, d_overlay_out: int, frame_id: int) -> int:
    """hs_submit_frame with the split-K scratch in the library's fixed device array (no
    allocation).  Returns HS_OK or HS_E_QUEUE_FULL; raises on any other status."""
    return _check(load().hs_submit_frame_static_scratch(app, d_frame, d_overlay_out, frame_id),
                  soft=(HS_E_QUEUE_FULL,))


def hs_poll_result(app: int):
    """Returns an hs_result, or None if no frame has finished."""
    r = hs_result()
    st = _check(load().hs_poll_result(app, C.byref(r)), soft=(HS_E_NOT_READY,))
    return r if st == HS_OK else None


def hs_wait_result(app: int, timeout_ns: int = 10_000_000_000):
    """Returns an hs_result, or None on time-out."""
    r = hs_result()
    st = _check(load().hs_wait_result(app, C.byref(r), timeout_ns), soft=(HS_E_NOT_READY,))
    return r if st == HS_OK else None


def hs_submit_batch(app: int, d_frames, d_overlay_outs, frame_id: int) -> int:
    """d_frames / d_overlay_outs: sequences of device pointers (ints), one per stream.
    Returns HS_OK or HS_E_QUEUE_FULL; raises on any other status."""
    n = len(d_frames)
    fr = (C.c_void_p * n)(*[int(x) for x in d_frames])
    ou = (C.c_void_p * n)(*[int(x) for x in d_overlay_outs])
    return _check(load().hs_submit_batch(app, fr, ou, frame_id), soft=(HS_E_QUEUE_FULL,))


def hs_submit_batch_after(app: int, d_frames, d_overlay_outs, frame_id: int, hip_event: int) -> int:
    """As hs_submit_batch, with stage 1 ordered behind a HIP event (its handle as an integer, e.g.
    ``torch.cuda.Event.cuda_event``) that the caller recorded after producing the frames."""
    n = len(d_frames)
    fr = (C.c_void_p * n)(*[int(x) for x in d_frames])
    ou = (C.c_void_p * n)(*[int(x) for x in d_overlay_outs])
    return _check(load().hs_submit_batch_after(app, fr, ou, frame_id, hip_event),
                  soft=(HS_E_QUEUE_FULL,))


def hs_poll_batch(app: int, batch: int):
    """Returns a list of `batch` hs_result (stream order), or None if nothing has finished."""
    r = (hs_result * batch)()
    st = _check(load().hs_poll_batch(app, r), soft=(HS_E_NOT_READY,))
    return list(r) if st == HS_OK else None


def hs_wait_batch(app: int, batch: int, timeout_ns: int = 10_000_000_000):
    """Returns a list of `batch` hs_result (stream order), or None on time-out."""
    r = (hs_result * batch)()
    st = _check(load().hs_wait_batch(app, r, timeout_ns), soft=(HS_E_NOT_READY,))
    return list(r) if st == HS_OK else None


def hs_create_group(ctx: int, members) -> int:
    """members: application handles (ints), in layer order. Returns the group handle."""
    n = len(members)
    arr = (C.c_void_p * n)(*[int(m) for m in members])
    out = C.c_void_p()
    _check(load().hs_create_group(ctx, arr, n, C.byref(out)))
    return out.value


def hs_destroy_group(group: int) -> None:
    _check(load().hs_destroy_group(group))


def hs_submit_group(group: int, d_frame: int, d_overlay_out: int, frame_id: int) -> int:
    """Returns HS_OK or HS_E_QUEUE_FULL; raises on any other status."""
    return _check(load().hs_submit_group(group, d_frame, d_overlay_out, frame_id),
                  soft=(HS_E_QUEUE_FULL,))


def hs_poll_group(group: int, n_members: int):
    """Returns a list of n_members hs_result (member order), or None if nothing has finished."""
    r = (hs_result * n_members)()
    st = _check(load().hs_poll_group(group, r), soft=(HS_E_NOT_READY,))
    return list(r) if st == HS_OK else None


def hs_wait_group(group: int, n_members: int, timeout_ns: int = 10_000_000_000):
    """Returns a list of n_members hs_result (member order), or None on time-out."""
    r = (hs_result * n_members)()
    st = _check(load().hs_wait_group(group, r, timeout_ns), soft=(HS_E_NOT_READY,))
    return list(r) if st == HS_OK else None


def hs_create_mux(app: int, batch: int) -> int:
    out = C.c_void_p()
    _check(load().hs_create_mux(app, batch, C.byref(out)))
    return out.value


def hs_destroy_mux(mux: int) -> None:
    _check(load().hs_destroy_mux(mux))


def hs_mux_submit(mux: int, stream: int, d_frame: int, d_overlay_out: int, frame_id: int) -> int:
    """Returns HS_OK or HS_E_QUEUE_FULL; raises on any other status."""
    return _check(load().hs_mux_submit(mux, stream, d_frame, d_overlay_out, frame_id),
                  soft=(HS_E_QUEUE_FULL,))


def hs_mux_poll(mux: int, stream: int):
    """Returns the stream's next hs_result, or None if none has finished."""
    r = hs_result()
    st = _check(load().hs_mux_poll(mux, stream, C.byref(r)), soft=(HS_E_NOT_READY,))
    return r if st == HS_OK else None


def hs_mux_wait(mux: int, stream: int, timeout_ns: int = 10_000_000_000):
    """Returns the stream's next hs_result, or None on time-out."""
    r = hs_result()
    st = _check(load().hs_mux_wait(mux, stream, C.byref(r), timeout_ns), soft=(HS_E_NOT_READY,))
    return r if st == HS_OK else None


def hs_run_feeds(feeds, fps: float, n_frames: int):
    """feeds: dicts with app (int), group (int) or mux (int) + mux_stream, frames and outs (lists, one entry per distinct
    frame / output, each a sequence of `batch` device pointers), results_per_frame, cpu (-1: no
    pin).  Returns (results, dropped, lateness_ns, elapsed_s): per feed the list of collected frames, each a
    list of results_per_frame hs_result; the number of dropped frames; the submit lateness of
    every frame in ns (zeros when fps == 0); the run's wall time in seconds, taken inside the
    library."""
    n = len(feeds)
    arr = (hs_feed * n)()
    keep, res_bufs, late_bufs = [], [], []
    for i, f in enumerate(feeds):
        batch = len(f["frames"][0])
        fr = (C.c_void_p * (len(f["frames"]) * batch))(*[int(p) for row in f["frames"] for p in row])
        ou = (C.c_void_p * (len(f["outs"]) * batch))(*[int(p) for row in f["outs"] for p in row])
        keep += [fr, ou]
        arr[i].app = f.get("app") or None
        arr[i].group = f.get("group") or None
        arr[i].mux = f.get("mux") or None
        arr[i].mux_stream = int(f.get("mux_stream", 0))
        arr[i].d_frames = C.cast(fr, C.c_void_p)
        arr[i].d_outs = C.cast(ou, C.c_void_p)
        arr[i].n_frames, arr[i].n_outs, arr[i].batch = len(f["frames"]), len(f["outs"]), batch
        arr[i].results_per_frame = int(f["results_per_frame"])
        arr[i].cpu = int(f.get("cpu", -1))
        res_bufs.append((hs_result * (n_frames * arr[i].results_per_frame))())
        late_bufs.append((C.c_int64 * n_frames)())
    res_ptrs = (C.c_void_p * n)(*[C.addressof(b) for b in res_bufs])
    late_ptrs = (C.c_void_p * n)(*[C.addressof(b) for b in late_bufs])
    dropped = (C.c_int * n)()
    elapsed = C.c_double()
    _check(load().hs_run_feeds(arr, n, float(fps), n_frames, res_ptrs, dropped, late_ptrs,
                               C.byref(elapsed)))
    results = []
    for i in range(n):
        per = arr[i].results_per_frame
        done = n_frames - dropped[i]
        results.append([[res_bufs[i][k * per + j] for j in range(per)] for k in range(done)])
    return results, list(dropped), [list(b) for b in late_bufs], elapsed.value


def hs_latency_metrics_compute(latencies, trim: bool = True) -> dict:
    x = np.ascontiguousarray(latencies, dtype=np.float64)
    m = hs_latency_metrics()
    _check(load().hs_latency_metrics_compute(x.ctypes.data, x.size, 1 if trim else 0,
                                             C.byref(m)))
    return {k: getattr(m, k) for k, _ in hs_latency_metrics._fields_}


def hs_mann_whitney_u(a, b) -> dict:
    """Two-sided Mann-Whitney U of two latency samples: {"u", "z", "significant"}."""
    x = np.ascontiguousarray(a, dtype=np.float64)
    y = np.ascontiguousarray(b, dtype=np.float64)
    r = hs_mwu()
    _check(load().hs_mann_whitney_u(x.ctypes.data, x.size, y.ctypes.data, y.size, C.byref(r)))
    return {"u": r.u, "z": r.z, "significant": bool(r.significant)}


def hs_set_cpu_affinity(app: int, cpu: int) -> None:
    _check(load().hs_set_cpu_affinity(app, int(cpu)))


def hs_device_copy(ctx: int, d_dst: int, d_src: int, nbytes: int) -> None:
    _check(load().hs_device_copy(ctx, d_dst, d_src, nbytes))


def hs_partition_copy(app: int, d_dst: int, d_src: int, nbytes: int, repeats: int = 10) -> float:
    """Seconds per copy of nbytes on the application's overlay stream (under its CU mask)."""
    sec = C.c_double()
    _check(load().hs_partition_copy(app, d_dst, d_src, nbytes, repeats, C.byref(sec)))
    return sec.value


def hs_set_launch_mode(app: int, mode: int) -> None:
    _check(load().hs_set_launch_mode(app, mode))


def hs_set_kernel_timing(app: int, enable: bool) -> None:
    _check(load().hs_set_kernel_timing(app, 1 if enable else 0))


def hs_get_kernel_times(app: int) -> list:
    buf = (hs_kernel_time * 16)()
    n = C.c_int()
    _check(load().hs_get_kernel_times(app, buf, 16, C.byref(n)))
    return [{"name": buf[i].name.decode(), "launches": buf[i].launches,
             "total_ms": buf[i].total_ms, "flops": buf[i].flops, "bytes": buf[i].bytes}
            for i in range(min(n.value, 16))]
