"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library never does.  The arithmetic lives in ``idfo.c`` (dense
layer-by-layer network and the scalar event-by-event streaming scheme, both in
double / int64) and in ``eager.py`` (the paper-literal eager scheme for tiny
nets).  This file only marshals numpy arrays into that C library.

Parity status: pinned by tests/test_oracle_*.py (closed forms, a library
convolution, brute force, the paper's invariants and its Fig. 1 figure of 7
stored activations).  The paper prints no worked numeric example, so absolute
output values are pinned only through those agreements.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libidfo.so")
_lib = None

_ACT = {"none": 0, "relu": 1, "relu_shr_clamp": 2}
_KIND = {"conv": 0, "maxpool": 1}


class _Layer(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("kind", "c_in", "c_out", "k_h", "k_w", "s_h", "s_w", "p_h", "p_w", "act", "shr", "clamp_hi")]


def build(force: bool = False) -> str:
    """Compile idfo.c with gcc into oracle/libidfo.so."""
    srcs = [os.path.join(_HERE, f) for f in ("idfo.c", "idfo_body.inc", "idfo.h")]
    if (not force and os.path.exists(_LIB_PATH)
            and all(os.path.getmtime(_LIB_PATH) >= os.path.getmtime(s) for s in srcs)):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", _LIB_PATH, srcs[0], "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB_PATH)
        L.idfo_round_bf16.restype = C.c_double
        L.idfo_round_bf16.argtypes = [C.c_double]
        L.idfo_out_size.restype = C.c_int
        for sfx in ("f64", "i64"):
            getattr(L, f"idfo_stream_new_{sfx}").restype = C.c_void_p
            getattr(L, f"idfo_stream_free_{sfx}").argtypes = [C.c_void_p]
            getattr(L, f"idfo_stream_push_{sfx}").argtypes = [C.c_void_p, C.c_void_p, C.c_int]
            getattr(L, f"idfo_stream_ready_{sfx}").restype = C.c_int64
            getattr(L, f"idfo_stream_ready_{sfx}").argtypes = [C.c_void_p]
            getattr(L, f"idfo_stream_take_{sfx}").restype = C.c_int64
            getattr(L, f"idfo_stream_take_{sfx}").argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
            getattr(L, f"idfo_stream_stats_{sfx}").argtypes = [C.c_void_p] + [C.c_void_p] * 4
            getattr(L, f"idfo_stream_head_{sfx}").restype = C.c_int64
            getattr(L, f"idfo_stream_head_{sfx}").argtypes = [C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def round_bf16(v: float) -> float:
    return float(lib().idfo_round_bf16(float(v)))


def out_size(n, k, s, p):
    t = n + 2 * p - k
    return 0 if t < 0 else t // s + 1


def layer_shapes(layers, in_h, in_w):
    """[(H_o, W_o, C_out)] per layer (H_o = 0 for an unbounded stream)."""
    shapes = []
    h, w = in_h, in_w
    for L in layers:
        h = out_size(h, L["k_h"], L["s_h"], L["p_h"]) if in_h else 0
        w = out_size(w, L["k_w"], L["s_w"], L["p_w"])
        shapes.append((h, w, L["c_out"]))
    return shapes


def _pack_layers(layers):
    arr = (_Layer * len(layers))()
    for i, L in enumerate(layers):
        arr[i] = _Layer(_KIND[L["kind"]], L["c_in"], L["c_out"], L["k_h"], L["k_w"], L["s_h"], L["s_w"],
                        L["p_h"], L["p_w"], _ACT[L.get("act", "none")], L.get("shr", 0), L.get("clamp_hi", 0))
    return arr


def _pack_ptrs(arrays, dtype):
    """ctypes pointer table over per-layer arrays (None -> NULL); keeps the arrays alive."""
    keep = [None if a is None else np.ascontiguousarray(a, dtype=dtype) for a in arrays]
    tbl = (C.c_void_p * len(keep))(*[None if a is None else a.ctypes.data for a in keep])
    return tbl, keep


def _flavour(integer):
    return ("i64", np.int64) if integer else ("f64", np.float64)


def dense(layers, x, weights, biases=None, *, integer=False, emit_round=None, return_layers=False):
    """The conventional layer-by-layer network on one sample x [H][W][C0].

    emit_round='bf16' rounds every activation handed from one layer to the next
    (not the last layer's) to bfloat16, as the bf16 GPU configuration does.
    """
    sfx, dt = _flavour(integer)
    x = np.ascontiguousarray(x, dtype=dt)
    H, W, C0 = x.shape
    shapes = layer_shapes(layers, H, W)
    biases = biases if biases is not None else [None] * len(layers)
    wt, wkeep = _pack_ptrs(weights, dt)
    bt, bkeep = _pack_ptrs(biases, dt)
    outs = [np.empty(s, dtype=dt) for s in shapes] if return_layers else None
    lt = (C.c_void_p * len(layers))(*[o.ctypes.data for o in outs]) if return_layers else None
    out = np.empty(shapes[-1], dtype=dt)
    rc = getattr(lib(), f"idfo_dense_{sfx}")(
        _pack_layers(layers), len(layers), H, W, C0, C.c_void_p(x.ctypes.data), wt, bt,
        1 if emit_round == "bf16" else 0, C.c_void_p(out.ctypes.data), lt)
    if rc != 0:
        raise ValueError("inconsistent layer description")
    del wkeep, bkeep
    return (out, outs) if return_layers else out


class Stream:
    """One stream of the paper's scheme: scalar events, rolling K_h-row state per layer."""

    def __init__(self, layers, in_h, in_w, in_c, weights, biases=None, *, integer=False,
                 emit_round=None, avg_head=False):
        self._sfx, self._dt = _flavour(integer)
        self.layers = layers
        self.in_w, self.in_c = in_w, in_c
        shapes = layer_shapes(layers, in_h, in_w)
        self.out_w, self.out_c = shapes[-1][1], shapes[-1][2]
        biases = biases if biases is not None else [None] * len(layers)
        self._wt, self._wkeep = _pack_ptrs(weights, self._dt)
        self._bt, self._bkeep = _pack_ptrs(biases, self._dt)
        self._h = getattr(lib(), f"idfo_stream_new_{self._sfx}")(
            _pack_layers(layers), len(layers), in_h, in_w, in_c, self._wt, self._bt,
            1 if emit_round == "bf16" else 0, 1 if avg_head else 0)
        if not self._h:
            raise ValueError("inconsistent layer description")

    def push(self, rows):
        rows = np.ascontiguousarray(rows, dtype=self._dt).reshape(-1, self.in_w, self.in_c)
        rc = getattr(lib(), f"idfo_stream_push_{self._sfx}")(self._h, rows.ctypes.data, rows.shape[0])
        if rc != 0:
            raise RuntimeError(f"oracle stream error {rc}: more than K_h rows of a layer were live")

    def ready(self) -> int:
        return int(getattr(lib(), f"idfo_stream_ready_{self._sfx}")(self._h))

    def take(self, max_rows=None):
        n = self.ready() if max_rows is None else min(self.ready(), max_rows)
        out = np.empty((n, self.out_w, self.out_c), dtype=self._dt)
        got = getattr(lib(), f"idfo_stream_take_{self._sfx}")(self._h, out.ctypes.data, n)
        assert got == n
        return out

    def stats(self):
        n = len(self.layers)
        ev = np.zeros(n, dtype=np.uint64)
        macs = np.zeros(n, dtype=np.uint64)
        peak_rows = np.zeros(n, dtype=np.int32)
        peak_cells = C.c_int64(0)
        getattr(lib(), f"idfo_stream_stats_{self._sfx}")(
            self._h, ev.ctypes.data, macs.ctypes.data, peak_rows.ctypes.data,
            C.cast(C.byref(peak_cells), C.c_void_p))
        return dict(events_in=ev, macs=macs, peak_rows=peak_rows, peak_cells=int(peak_cells.value))

    def head(self):
        mean = np.zeros(self.out_c, dtype=np.float64)
        rows = getattr(lib(), f"idfo_stream_head_{self._sfx}")(self._h, mean.ctypes.data)
        return int(rows), mean

    def close(self):
        if self._h:
            getattr(lib(), f"idfo_stream_free_{self._sfx}")(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def stream_run(wl_layers, x, weights, biases=None, *, seg_rows=1, integer=False, emit_round=None):
    """Feed one sample x [H][W][C0] through a Stream seg_rows rows at a time.

    Returns (output [H_o][W_o][C_o], stats dict)."""
    H, W, C0 = x.shape
    s = Stream(wl_layers, H, W, C0, weights, biases, integer=integer, emit_round=emit_round)
    chunks = []
    for r in range(0, H, seg_rows):
        s.push(x[r:r + seg_rows])
        if s.ready():
            chunks.append(s.take())
    st = s.stats()
    s.close()
    dt = np.int64 if integer else np.float64
    out = np.concatenate(chunks, axis=0) if chunks else np.empty((0, s.out_w, s.out_c), dtype=dt)
    return out, st


def head_units(out_rows, weights, bias=None):
    """Fully connected output units over the last layer's map (Sec. 4: the class units whose values
    settle as rows are presented): bias plus the weighted sum of the rows completed so far.
    out_rows [n][W][C] = the first n rows of the last layer's output; weights [K][H][W][C]."""
    o = np.asarray(out_rows, dtype=np.float64)
    w = np.asarray(weights, dtype=np.float64)[:, :o.shape[0]]
    v = np.tensordot(w, o, axes=([1, 2, 3], [0, 1, 2]))
    return v if bias is None else v + np.asarray(bias, dtype=np.float64)
