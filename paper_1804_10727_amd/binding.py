"""ctypes binding of libidf.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

IDF_OK, IDF_EINVAL, IDF_ENOMEM, IDF_ESTATE, IDF_EDEVICE, IDF_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
PREC = {"f32": 0, "bf16": 1, "i8": 2}
KIND = {"conv": 0, "maxpool": 1}
ACT = {"none": 0, "relu": 1, "relu_shr_clamp": 2}

EXPORTS = ["idf_create_net", "idf_create_net_columnwise", "idf_destroy_net", "idf_query_sizes", "idf_open_streams", "idf_open_streams_static", "idf_close_streams",
           "idf_push_segment", "idf_set_push_batching", "idf_read_outputs", "idf_reset_streams", "idf_get_stats", "idf_count_issued_macs", "idf_get_issued_macs", "idf_set_event_path", "idf_rows_pushed",
           "idf_layer_kernel", "idf_last_error", "idf_profile_begin", "idf_profile_end", "idf_enable_head",
           "idf_read_head", "idf_query_head_units_bytes", "idf_enable_head_units", "idf_read_head_units", "idf_push_pixels", "idf_query_eager_bytes", "idf_enable_eager", "idf_read_announced", "idf_read_announced_rows", "idf_eager_state_bytes", "idf_snapshot_bytes", "idf_snapshot", "idf_restore", "idf_create_net_volume", "idf_measure_peak"]


class IdfError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"idf error {code}: {text}")
        self.code = code


class _Layer(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("kind", "c_in", "c_out", "k_h", "k_w", "s_h", "s_w", "p_h", "p_w", "act", "shr", "clamp_hi")]


class _NetDesc(C.Structure):
    _fields_ = [("precision", C.c_int), ("in_h", C.c_int), ("in_w", C.c_int), ("in_c", C.c_int),
                ("n_layers", C.c_int), ("layers", C.POINTER(_Layer))]


class _Layer3d(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("c_in", "c_out", "k_d", "k_h", "k_w", "s_d", "s_h", "s_w", "p_d", "p_h", "p_w", "act", "shr", "clamp_hi")]


class _Net3dDesc(C.Structure):
    _fields_ = [("precision", C.c_int), ("in_d", C.c_int), ("in_h", C.c_int), ("in_w", C.c_int), ("in_c", C.c_int),
                ("n_layers", C.c_int), ("layers", C.POINTER(_Layer3d))]


class KernelProfile(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("launches", C.c_uint64), ("total_ms", C.c_double),
                ("algorithmic_bytes", C.c_double)]


class Sizes(C.Structure):
    _fields_ = [("workspace_bytes", C.c_size_t), ("weights_bytes", C.c_size_t),
                ("state_bytes_per_stream", C.c_size_t), ("handover_bytes_per_stream", C.c_size_t),
                ("retained_bytes_per_stream", C.c_size_t), ("transit_bytes_per_stream", C.c_size_t),
                ("output_bytes_per_stream", C.c_size_t), ("out_w", C.c_int), ("out_c", C.c_int),
                ("out_h", C.c_int64)]


def lib_path() -> str:
    return os.path.join(_HERE, "libidf.so")


def load_library():
    """Load libidf.so, building it first only if it is not there.  No fallback: without the
    HIP library nothing in this package works."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(lib_path()):
        from . import build as _build
        _build.build()
    # PyTorch ships its own copy of the HIP runtime (same soname).  Device pointers and streams
    # are only meaningful inside the runtime instance that made them, so that copy must be the
    # one this library binds to: import torch first, then the loader resolves our dependency
    # to the runtime already in the process.
    import torch  # noqa: F401
    L = C.CDLL(lib_path())
    L.idf_last_error.restype = C.c_char_p
    L.idf_layer_kernel.restype = C.c_char_p
    L.idf_layer_kernel.argtypes = [C.c_void_p, C.c_int]
    L.idf_create_net.argtypes = [C.POINTER(_NetDesc), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                 C.POINTER(C.c_void_p)]
    L.idf_create_net_columnwise.argtypes = L.idf_create_net.argtypes
    L.idf_create_net_volume.argtypes = [C.POINTER(_Net3dDesc), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                    C.POINTER(C.c_void_p)]
    L.idf_destroy_net.argtypes = [C.c_void_p]
    L.idf_query_sizes.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.POINTER(Sizes)]
    L.idf_open_streams.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_void_p, C.c_size_t,
                                   C.c_void_p, C.POINTER(C.c_void_p)]
    L.idf_open_streams_static.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_void_p, C.POINTER(C.c_void_p)]
    L.idf_close_streams.argtypes = [C.c_void_p]
    L.idf_push_segment.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int]
    L.idf_set_push_batching.argtypes = [C.c_void_p, C.c_int]
    L.idf_read_outputs.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int64,
                                   C.c_void_p, C.c_void_p]
    L.idf_reset_streams.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
    L.idf_get_stats.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    L.idf_get_issued_macs.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    L.idf_count_issued_macs.argtypes = [C.c_void_p, C.c_int]
    L.idf_set_event_path.argtypes = [C.c_void_p, C.c_int]
    L.idf_rows_pushed.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int64)]
    L.idf_enable_head.argtypes = [C.c_void_p]
    L.idf_query_head_units_bytes.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.idf_enable_head_units.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
    L.idf_read_head_units.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    L.idf_query_eager_bytes.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.idf_read_announced_rows.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    L.idf_eager_state_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t), C.c_void_p]
    L.idf_enable_eager.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t]
    L.idf_read_announced.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_void_p]
    L.idf_push_pixels.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int]
    L.idf_snapshot_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
    L.idf_snapshot.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    L.idf_restore.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    L.idf_read_head.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    L.idf_measure_peak.argtypes = [C.c_int, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double)]
    L.idf_profile_begin.argtypes = [C.c_void_p]
    L.idf_profile_end.argtypes = [C.c_void_p, C.c_int, C.POINTER(KernelProfile), C.POINTER(C.c_int)]
    _LIB = L
    return L


PEAK_KINDS = {"copy": 0, "fma_f32": 1, "mfma_f32": 2, "mfma_bf16": 3, "mfma_i8": 4}


def measure_peak(kind, buf):
    """idf_measure_peak on a torch uint8 device tensor: GB/s for "copy", tera-operations/s otherwise."""
    import torch
    rate = C.c_double()
    _check(load_library().idf_measure_peak(PEAK_KINDS[kind], C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                           C.c_void_p(torch.cuda.current_stream(buf.device).cuda_stream), C.byref(rate)))
    return rate.value


def _check(rc):
    if rc != IDF_OK:
        raise IdfError(rc, load_library().idf_last_error().decode())


def _ids(stream_ids):
    if stream_ids is None:
        return None, None
    a = np.ascontiguousarray(stream_ids, dtype=np.int32)
    return a, a.ctypes.data


class Net:
    """idf_create_net / idf_destroy_net."""

    def __init__(self, precision, in_h, in_w, in_c, layers, weights, biases=None, columnwise=False):
        L = load_library()
        self.precision = precision
        self.layers = layers
        n = len(layers)
        arr = (_Layer * n)()
        for i, d in enumerate(layers):
            arr[i] = _Layer(KIND[d["kind"]], d["c_in"], d["c_out"], d["k_h"], d["k_w"], d["s_h"], d["s_w"],
                            d["p_h"], d["p_w"], ACT[d.get("act", "none")], d.get("shr", 0), d.get("clamp_hi", 0))
        desc = _NetDesc(PREC[precision], in_h, in_w, in_c, n, arr)
        wdt = {"f32": np.float32, "bf16": np.uint16, "i8": np.int8}[precision]
        bdt = np.int32 if precision == "i8" else np.float32
        keep = []

        def table(arrays, dt):
            t = (C.c_void_p * n)()
            for i, a in enumerate(arrays):
                if a is None:
                    t[i] = None
                else:
                    a = np.ascontiguousarray(a, dtype=dt)
                    keep.append(a)
                    t[i] = a.ctypes.data
            return t
        wt = table(weights, wdt)
        bt = table(biases, bdt) if biases is not None else None
        h = C.c_void_p()
        create = L.idf_create_net_columnwise if columnwise else L.idf_create_net
        _check(create(C.byref(desc), wt, bt, C.byref(h)))
        self._h = h

    def query_sizes(self, n_streams, max_seg_rows=1, out_cap_rows=0) -> Sizes:
        s = Sizes()
        _check(load_library().idf_query_sizes(self._h, n_streams, max_seg_rows, out_cap_rows, C.byref(s)))
        return s

    def destroy(self):
        if self._h:
            _check(load_library().idf_destroy_net(self._h))
            self._h = None


class VolumeNet(Net):
    """idf_create_net_volume: volumes [slab][row][column][channel] presented slab by slab.  layers: dicts with c_in,
    c_out, k, s, p (triples over slab, row, column), act (, shr, clamp_hi); weights [c_out][c_in][k_d][k_h][k_w]."""

    def __init__(self, precision, in_d, in_h, in_w, in_c, layers, weights, biases=None):
        L = load_library()
        self.precision = precision
        self.layers = layers
        n = len(layers)
        arr = (_Layer3d * n)()
        for i, d in enumerate(layers):
            arr[i] = _Layer3d(d["c_in"], d["c_out"], *d["k"], *d["s"], *d["p"], ACT[d.get("act", "none")],
                              d.get("shr", 0), d.get("clamp_hi", 0))
        desc = _Net3dDesc(PREC[precision], in_d, in_h, in_w, in_c, n, arr)
        wdt = {"f32": np.float32, "bf16": np.uint16, "i8": np.int8}[precision]
        bdt = np.int32 if precision == "i8" else np.float32
        keep = []

        def table(arrays, dt):
            t = (C.c_void_p * n)()
            for i, a in enumerate(arrays):
                if a is None:
                    t[i] = None
                else:
                    a = np.ascontiguousarray(a, dtype=dt)
                    keep.append(a)
                    t[i] = a.ctypes.data
            return t
        wt = table(weights, wdt)
        bt = table(biases, bdt) if biases is not None else None
        h = C.c_void_p()
        _check(L.idf_create_net_volume(C.byref(desc), wt, bt, C.byref(h)))
        self._h = h


class Streams:
    """idf_open_streams ... idf_close_streams.  Tensors are torch CUDA tensors; only their
    data pointers cross the boundary."""

    def __init__(self, net: Net, n_streams, max_seg_rows=1, out_cap_rows=0, device="cuda:0", stream=None,
                 static_workspace=False):
        import torch
        self.net = net
        self.n_streams = n_streams
        self.max_seg_rows = max_seg_rows
        self.sizes = net.query_sizes(n_streams, max_seg_rows, out_cap_rows)
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            h = C.c_void_p()
            if static_workspace:        # idf_open_streams_static: the library's own array, nothing allocated here
                self.workspace = None
                _check(load_library().idf_open_streams_static(net._h, n_streams, max_seg_rows, out_cap_rows,
                                                              C.c_void_p(self.stream.cuda_stream), C.byref(h)))
                self._h = h
                self.out_dtype = torch.int32 if net.precision == "i8" else torch.float32
                return
            self.workspace = torch.empty(self.sizes.workspace_bytes + 256, dtype=torch.uint8, device=self.device)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            _check(load_library().idf_open_streams(net._h, n_streams, max_seg_rows, out_cap_rows,
                                                   C.c_void_p(self._ws_ptr), self.sizes.workspace_bytes,
                                                   C.c_void_p(self.stream.cuda_stream), C.byref(h)))
        self._h = h
        self.out_dtype = torch.int32 if net.precision == "i8" else torch.float32

    def push_segment(self, rows, stream_ids=None, n_rows=None):
        """rows: device tensor [n_ids][n_rows][in_w][in_c] (float32 / bfloat16 / int8)."""
        keep, ptr = _ids(stream_ids)
        n_ids = rows.shape[0] if stream_ids is None else len(keep)
        n_rows = rows.shape[1] if n_rows is None else n_rows
        assert rows.is_contiguous() and rows.is_cuda
        _check(load_library().idf_push_segment(self._h, ptr, n_ids, C.c_void_p(rows.data_ptr()), n_rows))

    def set_push_batching(self, k):
        _check(load_library().idf_set_push_batching(self._h, int(k)))

    def push_pixels(self, pixels, x0, stream_ids=None):
        """pixels: device tensor [n_ids][n_px][in_c] -- the next columns of the current row."""
        keep, ptr = _ids(stream_ids)
        assert pixels.is_contiguous()
        _check(load_library().idf_push_pixels(self._h, ptr, pixels.shape[0], C.c_void_p(pixels.data_ptr()), int(x0),
                                              int(pixels.shape[1])))

    def read_outputs(self, max_rows, stream_ids=None, n_ids=None, out=None):
        import torch
        keep, ptr = _ids(stream_ids)
        n_ids = (self.n_streams if n_ids is None else n_ids) if stream_ids is None else len(keep)
        if out is None:
            out = torch.empty((n_ids, max_rows, self.sizes.out_w, self.sizes.out_c), dtype=self.out_dtype,
                              device=self.device)
        first = np.zeros(n_ids, dtype=np.int64)
        cnt = np.zeros(n_ids, dtype=np.int32)
        _check(load_library().idf_read_outputs(self._h, ptr, n_ids, C.c_void_p(out.data_ptr()), max_rows,
                                               first.ctypes.data, cnt.ctypes.data))
        return out, first, cnt

    def reset(self, stream_ids=None, n_ids=None):
        keep, ptr = _ids(stream_ids)
        n_ids = (self.n_streams if n_ids is None else n_ids) if stream_ids is None else len(keep)
        _check(load_library().idf_reset_streams(self._h, ptr, n_ids))

    def get_stats(self, stream_id):
        n = len(self.net.layers)
        ev = np.zeros(n, dtype=np.uint64); macs = np.zeros(n, dtype=np.uint64); sb = np.zeros(n, dtype=np.uint64)
        _check(load_library().idf_get_stats(self._h, stream_id, ev.ctypes.data, macs.ctypes.data, sb.ctypes.data))
        return dict(events_in=ev, macs=macs, state_bytes=sb)

    def count_issued_macs(self, on=True):
        _check(load_library().idf_count_issued_macs(self._h, int(bool(on))))

    def set_event_path(self, events_per_kstep):
        _check(load_library().idf_set_event_path(self._h, int(events_per_kstep)))

    def get_issued_macs(self, stream_id):
        iss = np.zeros(len(self.net.layers), dtype=np.uint64)
        _check(load_library().idf_get_issued_macs(self._h, stream_id, iss.ctypes.data))
        return iss

    def rows_pushed(self, stream_id):
        r = C.c_int64()
        _check(load_library().idf_rows_pushed(self._h, stream_id, C.byref(r)))
        return r.value

    def snapshot(self, stream_id):
        """(device buffer, position) holding the stream's retained state."""
        import torch
        L = load_library()
        nb = C.c_size_t()
        _check(L.idf_snapshot_bytes(self._h, C.byref(nb)))
        buf = torch.empty(max(1, nb.value), dtype=torch.uint8, device=self.device)
        pos = (C.c_int64 * 3)()
        _check(L.idf_snapshot(self._h, stream_id, C.c_void_p(buf.data_ptr()), pos))
        return buf, tuple(pos)

    def restore(self, stream_id, buf, pos):
        arr = (C.c_int64 * 3)(*pos)
        _check(load_library().idf_restore(self._h, stream_id, C.c_void_p(buf.data_ptr()), arr))

    def enable_eager(self):
        """Eager emission: allocates the second workspace and switches the streams over."""
        import torch
        L = load_library()
        nb = C.c_size_t()
        _check(L.idf_query_eager_bytes(self.net._h, self.n_streams, self.max_seg_rows, C.byref(nb)))
        self._eager_ws = torch.empty(max(1, nb.value), dtype=torch.uint8, device=self.device)
        _check(L.idf_enable_eager(self._h, C.c_void_p(self._eager_ws.data_ptr()), nb.value))

    def read_announced(self, level, shape, stream_ids=None):
        """Announced map of a level (0 = input), [n][H][W][C]; shape = (H, W, C) of that level."""
        import torch
        keep, ptr = _ids(stream_ids)
        n = self.n_streams if stream_ids is None else len(keep)
        out = torch.empty((n,) + tuple(shape), dtype=torch.int32 if self.net.precision == "i8" else torch.float32,
                          device=self.device)
        _check(load_library().idf_read_announced(self._h, level, ptr, n, C.c_void_p(out.data_ptr())))
        return out

    def read_announced_rows(self, level, row_shape, max_rows, stream_ids=None):
        """Rows of a level that are still kept: (tensor [n][max_rows][W][C], first row [n], rows [n]);
        row_shape = (W, C) of that level."""
        import torch
        keep, ptr = _ids(stream_ids)
        n = self.n_streams if stream_ids is None else len(keep)
        out = torch.zeros((n, max_rows) + tuple(row_shape), dtype=torch.int32 if self.net.precision == "i8" else torch.float32,
                          device=self.device)
        first = np.zeros(n, dtype=np.int64); cnt = np.zeros(n, dtype=np.int32)
        _check(load_library().idf_read_announced_rows(self._h, level, ptr, n, C.c_void_p(out.data_ptr()), max_rows,
                                                      first.ctypes.data, cnt.ctypes.data))
        return out, first, cnt

    def eager_state_bytes(self):
        """(bytes of state and announced values retained per stream, rows kept per level)."""
        nb = C.c_size_t()
        rows = np.zeros(len(self.net.layers) + 1, dtype=np.int32)
        _check(load_library().idf_eager_state_bytes(self._h, C.byref(nb), rows.ctypes.data))
        return nb.value, rows

    def enable_head_units(self, weights, bias=None):
        """weights [n_units][out_h][out_w][out_c] (float32), bias [n_units] or None."""
        import torch
        L = load_library()
        w = np.ascontiguousarray(weights, dtype=np.float32)
        b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
        nb = C.c_size_t()
        _check(L.idf_query_head_units_bytes(self.net._h, self.n_streams, w.shape[0], C.byref(nb)))
        self._units_ws = torch.empty(max(1, nb.value), dtype=torch.uint8, device=self.device)
        self._n_units = int(w.shape[0])
        _check(L.idf_enable_head_units(self._h, w.shape[0], w.ctypes.data, None if b is None else b.ctypes.data,
                                       C.c_void_p(self._units_ws.data_ptr()), nb.value))

    def read_head_units(self, stream_ids=None):
        keep, ptr = _ids(stream_ids)
        n = self.n_streams if stream_ids is None else len(keep)
        vals = np.zeros((n, self._n_units), dtype=np.float64)
        rows = np.zeros(n, dtype=np.int64)
        _check(load_library().idf_read_head_units(self._h, ptr, n, vals.ctypes.data, rows.ctypes.data))
        return rows, vals

    def enable_head(self):
        _check(load_library().idf_enable_head(self._h))

    def read_head(self, stream_ids=None):
        """(rows averaged [n], mean [n][out_c]) of the averaging output units."""
        keep, ptr = _ids(stream_ids)
        n = self.n_streams if stream_ids is None else len(keep)
        mean = np.zeros((n, int(self.sizes.out_c)), dtype=np.float64)
        rows = np.zeros(n, dtype=np.int64)
        _check(load_library().idf_read_head(self._h, ptr, n, mean.ctypes.data, rows.ctypes.data))
        return rows, mean

    def profile_begin(self):
        _check(load_library().idf_profile_begin(self._h))

    def profile_end(self):
        arr = (KernelProfile * 64)()
        n = C.c_int()
        _check(load_library().idf_profile_end(self._h, 64, arr, C.byref(n)))
        return [dict(name=arr[i].name.decode(), launches=int(arr[i].launches), total_ms=float(arr[i].total_ms),
                     algorithmic_bytes=float(arr[i].algorithmic_bytes)) for i in range(n.value)]

    def layer_kernels(self):
        L = load_library()
        return [L.idf_layer_kernel(self._h, i).decode() for i in range(len(self.net.layers))]

    def close(self):
        if self._h:
            _check(load_library().idf_close_streams(self._h))
            self._h = None


def create_net(precision, in_h, in_w, in_c, layers, weights, biases=None) -> Net:
    return Net(precision, in_h, in_w, in_c, layers, weights, biases)


def open_streams(net, n_streams, **kw) -> Streams:
    return Streams(net, n_streams, **kw)


def _bf16_bits(a):
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return (u >> 16).astype(np.uint16)


def net_from_workload(wl, columnwise=False) -> Net:
    """Net from a workload dict (see the workloads module): only dtype marshalling."""
    prec = wl["precision"]
    if prec == "bf16":
        ws = [None if w is None else _bf16_bits(w) for w in wl["weights"]]
    else:
        ws = wl["weights"]
    return Net(prec, wl["in_h"], wl["in_w"], wl["in_c"], wl["layers"], ws, wl["biases"], columnwise=columnwise)


def input_tensor(wl, device="cuda:0"):
    """The workload's input as a device tensor of the net's input type: [streams][H][W][C]."""
    import torch
    x = wl["x"]
    if wl["precision"] == "bf16":
        return torch.from_numpy(np.ascontiguousarray(x)).to(device).to(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).to(device)
