"""Convenience wrapper used by tests and benchmarks: builds a library context from host weights
that follow the documented blob format (any object exposing ``shape``, ``layer_blobs`` and
``global_blob`` numpy arrays, e.g. weights generated into pinned memory).  Marshalling only.
"""
from __future__ import annotations

from typing import Optional

from . import binding as B


class Session:
    def __init__(self, target_w, draft_w=None, **cfg):
        self._keep = (target_w, draft_w)
        tw = B.make_host_weights([b.ctypes.data for b in target_w.layer_blobs], target_w.global_blob.ctypes.data)
        dw = None
        if draft_w is not None:
            dw = B.make_host_weights([b.ctypes.data for b in draft_w.layer_blobs], draft_w.global_blob.ctypes.data)
        self.target_shape = target_w.shape
        self.draft_shape = draft_w.shape if draft_w is not None else None
        self.ctx = B.spec_init(target_w.shape, self.draft_shape, tw, dw, **cfg)

    def close(self):
        if self.ctx:
            B.spec_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
