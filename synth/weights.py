"""Random-init weights in the host blob format described in ``synth.shapes``.

Values: every weight matrix ~ N(0, std^2) (default 0.02), every RMSNorm gain = 1 (the
benchmark workloads) or 1 + N(0, gain_std^2) (parity tests: a gain of exactly 1 would hide
a dropped or misplaced gain), from a counter-based generator (see ``gen.c``) keyed by (seed, tensor id, element index);
bf16 models are rounded to nearest-even once, here, so that the oracle and the HIP
library read the very same numbers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Callable, Dict, List, Optional

import numpy as np

from .shapes import ModelShape

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsynthgen.so")
_lib = None
_qtable = None


def build_lib(force: bool = False) -> str:
    """Compile gen.c with gcc (host only)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O3", "-march=x86-64-v2", "-shared", "-fPIC", "-pthread",
                               "-o", _SO, src])
    return _SO


def _load():
    global _lib, _qtable
    if _lib is None:
        build_lib()
        lib = ctypes.CDLL(_SO)
        lib.synth_fill_normal.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                                          ctypes.c_uint32, ctypes.c_uint32, ctypes.c_float,
                                          ctypes.c_float, ctypes.c_void_p, ctypes.c_int]
        lib.synth_fill_normal.restype = ctypes.c_int
        lib.synth_fill_const.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int,
                                         ctypes.c_float]
        lib.synth_fill_const.restype = ctypes.c_int
        lib.synth_philox4x32_10.argtypes = [ctypes.c_void_p] * 3
        lib.synth_philox4x32_10.restype = None
        from scipy.special import ndtri
        _qtable = np.ascontiguousarray(ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
                                       .astype(np.float32))
        _lib = lib
    return _lib


def philox4x32_10(ctr, key) -> np.ndarray:
    """One Philox block from the C generator (for its known-answer test)."""
    lib = _load()
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib.synth_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 (exact)."""
    return (a.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 bit patterns, nearest-even (data-format helper)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def fill_normal(dst: np.ndarray, seed: int, tid: int, std: float = 0.02, mean: float = 0.0,
                n_threads: Optional[int] = None) -> None:
    lib = _load()
    assert dst.flags["C_CONTIGUOUS"] and dst.dtype in (np.float32, np.uint16)
    nt = n_threads or min(16, os.cpu_count() or 1)
    rc = lib.synth_fill_normal(dst.ctypes.data, dst.size, 0 if dst.dtype == np.float32 else 1,
                               seed & 0xFFFFFFFF, tid & 0xFFFFFFFF, mean, std,
                               _qtable.ctypes.data, nt)
    assert rc == 0


def fill_const(dst: np.ndarray, value: float) -> None:
    lib = _load()
    rc = lib.synth_fill_const(dst.ctypes.data, dst.size, 0 if dst.dtype == np.float32 else 1, value)
    assert rc == 0


def _tid(layer: int, name: str) -> int:
    base = (layer + 1) * 1000           # layer -1 = globals
    if name in ("g1", "emb"):
        return base + 1
    if name in ("wqkv", "gf"):
        return base + 2
    if name in ("wo", "head"):
        return base + 3
    if name == "g2":
        return base + 4
    if name == "wr":
        return base + 5
    kind, e = name.split("_")
    return base + 10 + 3 * int(e) + {"w1": 0, "w3": 1, "w2": 2}[kind]


class HostModel:
    """Host-resident weights of one model: a list of layer blobs and one global blob.

    ``layer_blobs[l]`` / ``global_blob`` are 1-D numpy arrays (uint16 for bf16, float32
    for f32) possibly backed by pinned memory supplied through ``alloc``.  Several
    layers may alias one blob (``unique_layers``) when a benchmark needs the byte
    traffic of a large model without its full host footprint.
    """

    def __init__(self, shape: ModelShape, layer_blobs: List[np.ndarray], global_blob: np.ndarray,
                 keepalive=None):
        self.shape = shape
        self.layer_blobs = layer_blobs
        self.global_blob = global_blob
        self._keepalive = keepalive

    def layer(self, l: int, widen: bool = True) -> Dict[str, np.ndarray]:
        """Named tensors of layer ``l``; bf16 is widened to float32 when ``widen``."""
        lay, _ = self.shape.layer_layout()
        return self._views(self.layer_blobs[l], lay, widen)

    def globals(self, widen: bool = True) -> Dict[str, np.ndarray]:
        lay, _ = self.shape.global_layout()
        return self._views(self.global_blob, lay, widen)

    def _views(self, blob, lay, widen):
        out = {}
        for name, (off, shp) in lay.items():
            n = int(np.prod(shp))
            v = blob[off:off + n].reshape(shp)
            if widen and v.dtype == np.uint16:
                v = bf16_bits_to_f32(v)
            out[name] = v
        return out

    def draft_view(self, n_layers: int, attn_only: bool) -> "HostModel":
        """The draft: the first ``n_layers`` layers of this model (attention part only if
        ``attn_only``), sharing embedding, final norm and LM head.  No copy: the attention
        part is a prefix of each layer blob."""
        ds = self.shape.draft(n_layers, attn_only)
        n = ds.layer_layout()[1]
        return HostModel(ds, [b[:n] for b in self.layer_blobs[:n_layers]], self.global_blob,
                         keepalive=self)


def make_model(shape: ModelShape, seed: int = 0,
               alloc: Optional[Callable[[int, np.dtype], np.ndarray]] = None,
               unique_layers: Optional[int] = None, std: float = 0.02,
               n_threads: Optional[int] = None, gain_std: float = 0.0) -> HostModel:
    """Generate all weights of ``shape``.

    ``alloc(n_elems, dtype)`` returns a 1-D contiguous array to fill (default
    ``np.empty``); the HIP harness passes an allocator handing out pinned memory.
    ``unique_layers``: generate only that many distinct layer blobs and alias layer
    ``l`` to blob ``l % unique_layers``.
    ``gain_std``: RMSNorm gains are 1 + N(0, gain_std^2) instead of exactly 1.
    """
    np_dt = np.uint16 if shape.dtype == "bf16" else np.float32
    alloc = alloc or (lambda n, dt: np.empty(n, dtype=dt))
    lay, n_layer = shape.layer_layout()
    glay, n_glob = shape.global_layout()
    uniq = shape.n_layers if not unique_layers else min(unique_layers, shape.n_layers)

    def fill(blob, layout, layer):
        for name, (off, shp) in layout.items():
            n = int(np.prod(shp))
            v = blob[off:off + n]
            if name in ("g1", "g2", "gf"):
                if gain_std > 0.0:
                    fill_normal(v, seed, _tid(layer, name), std=gain_std, mean=1.0, n_threads=n_threads)
                else:
                    fill_const(v, 1.0)
            else:
                fill_normal(v, seed, _tid(layer, name), std=std, n_threads=n_threads)
            pad = blob[off + n: off + (n + 127) // 128 * 128]
            if pad.size:
                pad[:] = 0

    blobs = []
    for l in range(uniq):
        b = alloc(n_layer, np_dt)
        assert b.size == n_layer and b.dtype == np_dt
        fill(b, lay, l)
        blobs.append(b)
    layer_blobs = [blobs[l % uniq] for l in range(shape.n_layers)]
    g = alloc(n_glob, np_dt)
    fill(g, glay, -1)
    return HostModel(shape, layer_blobs, g)
