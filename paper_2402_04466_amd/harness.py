"""Small harness over the binding: PyTorch supplies device memory (workspace, frames,
overlay outputs); everything that computes runs inside libhs.

``AppStream`` is one application stream (paper Section III-A), ``GroupStream`` a multi-network
application (Section III-B); ``run_paced`` drives several
of them concurrently at a fixed frame rate, one submitting thread per stream, the way the
paper runs one process per application instance (Section V-B).
"""
from __future__ import annotations

import os
import threading
import time

import numpy as np
import torch

from . import api


class AppStream:
    def __init__(self, ctx: int, *, net: int, frame_w: int, frame_h: int, net_w: int, net_h: int,
                 blob: np.ndarray, palette: np.ndarray, queue_depth: int = 2,
                 net_fp32_input: bool = False, frame_pitch: int | None = None, mean: float = 0.5,
                 std: float = 0.25, threshold: float = 0.5, alpha: float = 0.5, batch: int = 1,
                 glyphs=None, marker_arm: int = 12, marker_half: int = 1, glyph_scale: int = 2,
                 device: str = "cuda:0"):
        self.ctx = ctx
        self.frame_w, self.frame_h = frame_w, frame_h
        self.frame_pitch = frame_pitch if frame_pitch is not None else (3 * frame_w + 15) // 16 * 16
        self.net_w, self.net_h = net_w, net_h
        self.device = torch.device(device)
        kw = dict(frame_w=frame_w, frame_h=frame_h, net_w=net_w, net_h=net_h, net=net,
                  weights=blob, palette=palette, frame_pitch=self.frame_pitch,
                  net_fp32_input=int(net_fp32_input), mean=mean, std=std, threshold=threshold,
                  alpha=alpha, queue_depth=queue_depth, batch=batch, glyphs=glyphs,
                  marker_arm=marker_arm, marker_half=marker_half, glyph_scale=glyph_scale)
        self.batch = batch
        need = api.hs_query_workspace(api.make_desc(**kw))
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        self._ws_off = base - self.workspace.data_ptr()
        self.workspace_bytes = need
        torch.cuda.synchronize(self.device)
        self.app = api.hs_create_app(ctx, api.make_desc(d_workspace=base, workspace_bytes=need, **kw))
        self.queue_depth = queue_depth
        self._held = {}

    # -- device buffers ---------------------------------------------------------------------
    def upload_frame(self, frame: np.ndarray) -> torch.Tensor:
        """HxWx3 uint8 host frame -> pitched device buffer (H x pitch bytes)."""
        h, w, _ = frame.shape
        assert (w, h) == (self.frame_w, self.frame_h)
        host = np.zeros((h, self.frame_pitch), dtype=np.uint8)
        host[:, :3 * w] = frame.reshape(h, 3 * w)
        return torch.from_numpy(host).to(self.device)

    def new_output(self) -> torch.Tensor:
        return torch.zeros((self.frame_h, self.frame_pitch), dtype=torch.uint8, device=self.device)

    # -- hot path ---------------------------------------------------------------------------
    def submit(self, d_frame: torch.Tensor, d_out: torch.Tensor, frame_id: int) -> int:
        st = api.hs_submit_frame(self.app, d_frame.data_ptr(), d_out.data_ptr(), frame_id)
        if st == api.HS_OK:
            self._held[frame_id] = (d_frame, d_out)      # keep alive until polled
        return st

    def submit_batch(self, d_frames, d_outs, frame_id: int) -> int:
        """One frame per stream of a batched application (lists of device tensors)."""
        st = api.hs_submit_batch(self.app, [t.data_ptr() for t in d_frames],
                                 [t.data_ptr() for t in d_outs], frame_id)
        if st == api.HS_OK:
            self._held[frame_id] = (list(d_frames), list(d_outs))
        return st

    def wait_batch(self, timeout_s: float = 30.0):
        rs = api.hs_wait_batch(self.app, self.batch, int(timeout_s * 1e9))
        if rs is None:
            raise TimeoutError("no result within %.1f s" % timeout_s)
        self._held.pop(rs[0].frame_id, None)
        return rs

    def poll_batch(self):
        rs = api.hs_poll_batch(self.app, self.batch)
        if rs is not None:
            self._held.pop(rs[0].frame_id, None)
        return rs

    def poll(self):
        r = api.hs_poll_result(self.app)
        if r is not None:
            self._held.pop(r.frame_id, None)
        return r

    def wait(self, timeout_s: float = 30.0):
        r = api.hs_wait_result(self.app, int(timeout_s * 1e9))
        if r is None:
            raise TimeoutError("no result within %.1f s" % timeout_s)
        self._held.pop(r.frame_id, None)
        return r

    # -- read-back (tests, smoke) -----------------------------------------------------------
    def _view(self, ptr: int, nbytes: int) -> torch.Tensor:
        off = ptr - self.workspace.data_ptr()
        assert 0 <= off and off + nbytes <= self.workspace.numel(), "pointer outside workspace"
        return self.workspace[off:off + nbytes]

    def fetch(self, r, d_out: torch.Tensor | None = None) -> dict:
        """Copy one frame's device results to host NumPy arrays."""
        n = r.map_w * r.map_h
        out = {"argmax_idx": np.array(list(r.argmax_idx), dtype=np.int32),
               "present": np.array(list(r.present), dtype=np.uint8),
               "peak": np.array(list(r.peak), dtype=np.float32)}
        out["logits"] = self._view(r.d_logits, 32 * n).view(torch.float32).cpu().numpy().reshape(
            8, r.map_h, r.map_w)
        out["heat"] = self._view(r.d_heat, 32 * n).view(torch.float32).cpu().numpy().reshape(
            8, r.map_h, r.map_w)
        out["mask"] = self._view(r.d_mask, 8 * n).cpu().numpy().reshape(8, r.map_h, r.map_w)
        pitch = r.net_input_pitch_bytes
        rows = self._view(r.d_net_input, pitch * (self.net_h - 1) + 8 * self.net_w)
        rows = torch.nn.functional.pad(rows, (0, pitch * self.net_h - rows.numel()))
        ni = rows.view(self.net_h, pitch)[:, :8 * self.net_w].contiguous().view(torch.float16)
        out["net_input"] = ni.cpu().numpy().reshape(self.net_h, self.net_w, 4)
        if r.d_net_input_f32:
            out["net_input_f32"] = self._view(
                r.d_net_input_f32, 12 * self.net_w * self.net_h).view(torch.float32).cpu().numpy(
            ).reshape(3, self.net_h, self.net_w)
        if d_out is not None:
            out["overlay"] = d_out.cpu().numpy()[:, :3 * self.frame_w].reshape(
                self.frame_h, self.frame_w, 3)
        return out

    def state(self, r, stream: int = 0):
        return api.hs_get_state(self.app, r.map_h, r.map_w, stream=stream)

    def features(self, r, stream: int = 0):
        return api.hs_get_features(self.app, r.map_h, r.map_w, stream=stream)

    def close(self):
        if self.app:
            api.hs_destroy_app(self.app)
            self.app = None
            self._held.clear()


class GroupStream:
    """A multi-network application (paper Section III-B): AppStream members that all look at the
    same frame and share one overlay launch.  Offers the batch-style calls run_paced uses; a
    result is the list of the members' hs_result for one frame (member order)."""

    def __init__(self, ctx: int, members):
        self.members = list(members)
        self.group = api.hs_create_group(ctx, [m.app for m in self.members])
        self.batch = 1
        self._held = {}
        m0 = self.members[0]
        self.frame_w, self.frame_h, self.frame_pitch = m0.frame_w, m0.frame_h, m0.frame_pitch
        self.upload_frame, self.new_output = m0.upload_frame, m0.new_output

    def submit(self, d_frame: torch.Tensor, d_out: torch.Tensor, frame_id: int) -> int:
        st = api.hs_submit_group(self.group, d_frame.data_ptr(), d_out.data_ptr(), frame_id)
        if st == api.HS_OK:
            self._held[frame_id] = (d_frame, d_out)
        return st

    def submit_batch(self, d_frames, d_outs, frame_id: int) -> int:
        return self.submit(d_frames[0], d_outs[0], frame_id)

    def poll_batch(self):
        rs = api.hs_poll_group(self.group, len(self.members))
        if rs is not None:
            self._held.pop(rs[0].frame_id, None)
        return rs

    def wait_batch(self, timeout_s: float = 30.0):
        rs = api.hs_wait_group(self.group, len(self.members), int(timeout_s * 1e9))
        if rs is None:
            raise TimeoutError("no result within %.1f s" % timeout_s)
        self._held.pop(rs[0].frame_id, None)
        return rs

    def close(self):
        if self.group:
            api.hs_destroy_group(self.group)
            self.group = None
        for m in self.members:
            m.close()
        self._held.clear()


def _feeds(streams, frames, outputs, pin_cpus, muxes=None):
    """One feed per application, or, for an application behind a mux (muxes[i] not None), one
    feed per stream of its batch.  Returns the feeds and, per application, the indices of its
    feeds."""
    feeds, owner = [], []
    for i, s in enumerate(streams):
        if muxes is not None and muxes[i] is not None:
            idx = []
            for j in range(s.batch):
                idx.append(len(feeds))
                feeds.append({"mux": muxes[i], "mux_stream": j, "results_per_frame": 1,
                              "frames": [[row[j].data_ptr()] for row in frames[i]],
                              "outs": [[row[j].data_ptr()] for row in outputs[i]],
                              "cpu": -1 if pin_cpus is None else pin_cpus[i]})
            owner.append(idx)
            continue
        owner.append([len(feeds)])
        f = {"frames": [[t.data_ptr() for t in row] for row in frames[i]],
             "outs": [[t.data_ptr() for t in row] for row in outputs[i]],
             "cpu": -1 if pin_cpus is None else pin_cpus[i]}
        if isinstance(s, GroupStream):
            f["group"], f["results_per_frame"] = s.group, len(s.members)
        else:
            f["app"], f["results_per_frame"] = s.app, s.batch
        feeds.append(f)
    return feeds, owner


def _regroup(per_feed, owner):
    """Per application: per frame, the results of all its streams (a muxed application's feeds
    are merged frame by frame; frames that some stream dropped are left out)."""
    out = []
    for idx in owner:
        if len(idx) == 1:
            out.append(per_feed[idx[0]])
        else:
            n = min(len(per_feed[j]) for j in idx)
            out.append([[per_feed[j][k][0] for j in idx] for k in range(n)])
    return out


def run_paced(streams, frames, fps: float, outputs, pin_cpus=None, n_frames=None,
              with_lateness: bool = False, muxes=None):
    """Frame k of every application is submitted at t0 + k/fps by the library's native driver
    (one submitting thread per application, absolute deadlines: `hs_run_feeds`), the way the
    paper runs one process per application instance (Section V-B).  ``frames[i][k]`` /
    ``outputs[i][q]`` are lists with one device tensor per stream of application i (length
    ``batch``; a group takes one); frame k uses ``frames[i][k % len]`` and
    ``outputs[i][k % len]``.  Returns, per application, the list of per-frame result lists (one
    hs_result per stream, or per member of a group), plus the number of frames dropped because
    the queue was full.  ``pin_cpus[i]``: CPU core the submitting thread of application i pins
    itself to.  ``muxes[i]``: a mux handle when the streams of batched application i submit on their
    own, one thread per stream (their results are merged per frame again)."""
    n = n_frames if n_frames is not None else max(len(f) for f in frames)
    feeds, owner = _feeds(streams, frames, outputs, pin_cpus, muxes)
    results, dropped, late, _ = api.hs_run_feeds(feeds, fps, n)
    results = _regroup(results, owner)
    dropped = [sum(dropped[j] for j in idx) for idx in owner]
    late = [[v for j in idx for v in late[j]] for idx in owner]
    return (results, dropped, late) if with_lateness else (results, dropped)


def run_back_to_back(streams, frames, outputs, n_frames: int):
    """Every application submits n_frames frames as fast as its queue takes them (native driver,
    one thread each).  Returns the per-application results as run_paced does and the wall time
    of the run in seconds, measured inside the library from the start of the submitting threads
    to the collection of the last result (all GPU work of the run is complete then)."""
    feeds, owner = _feeds(streams, frames, outputs, None)
    results, _, _, elapsed = api.hs_run_feeds(feeds, 0.0, n_frames)
    return _regroup(results, owner), elapsed
