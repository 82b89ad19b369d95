"""Host-only checks of the HIP library: it loads, exports the declared C ABI, validates
network descriptions and reports sizes.  No GPU needed (no compute call is made)."""
import os
import re

import numpy as np
import pytest

import paper_1804_10727_amd as idf
from paper_1804_10727_amd import binding
import workloads as wl_mod
from workloads import conv, maxpool

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_every_declared_symbol():
    L = idf.load_library()
    header = open(os.path.join(ROOT, "include", "idf.h")).read()
    declared = set(re.findall(r"\b(idf_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_create_net_validation():
    w = [np.zeros((4, 2, 3, 3), np.float32)]
    with pytest.raises(idf.IdfError) as e:
        idf.Net("f32", 8, 8, 3, [conv(2, 4, 3, 3)], w)             # channel chain
    assert e.value.code == binding.IDF_EINVAL
    with pytest.raises(idf.IdfError) as e:
        idf.Net("f32", 0, 1, 2, [conv(2, 4, 3, 1, p_h=1)], [np.zeros((4, 2, 3, 1), np.float32)])   # unbounded + padding
    assert e.value.code == binding.IDF_EINVAL
    with pytest.raises(idf.IdfError) as e:
        idf.Net("f32", 2, 8, 2, [conv(2, 4, 3, 3)], w)             # kernel larger than input
    assert e.value.code == binding.IDF_EINVAL
    with pytest.raises(idf.IdfError) as e:
        idf.Net("f32", 8, 8, 2, [conv(2, 4, 3, 3, act="relu_shr_clamp", shr=4, clamp_hi=15)], w)
    assert e.value.code == binding.IDF_EUNSUPPORTED
    with pytest.raises(idf.IdfError) as e:                          # int8 events need the clamp
        idf.Net("i8", 8, 8, 2, [conv(2, 4, 3, 3), conv(4, 4, 1, 1)],
                [np.zeros((4, 2, 3, 3), np.int8), np.zeros((4, 4, 1, 1), np.int8)])
    assert e.value.code == binding.IDF_EUNSUPPORTED
    bad_pool = maxpool(4); bad_pool["k_h"] = 3
    with pytest.raises(idf.IdfError):
        idf.Net("f32", 8, 8, 2, [conv(2, 4, 3, 3), bad_pool], w + [None])
    with pytest.raises(idf.IdfError):
        idf.Net("f32", 8, 8, 2, [conv(2, 4, 3, 3)], [None])        # missing weights
    net = idf.Net("f32", 8, 8, 2, [conv(2, 4, 3, 3)], w)
    net.destroy()


# retained state per stream the build is held to: K_h rows of c (4 bytes) per conv layer plus
# one held row of activations per pool
def bound_bytes(wl):
    eb = {"f32": 4, "bf16": 2, "i8": 1}[wl["precision"]]
    h, w = wl["in_h"], wl["in_w"]
    total = 0
    for L in wl["layers"]:
        w_in = w
        h = wl_mod.out_size(h, L["k_h"], L["s_h"], L["p_h"])
        w = wl_mod.out_size(w, L["k_w"], L["s_w"], L["p_w"])
        total += L["k_h"] * w * L["c_out"] * 4 if L["kind"] == "conv" else w_in * L["c_out"] * eb
    return total


@pytest.mark.parametrize("cfg,kw", [(1, dict(streams=1, length=64)), (2, dict(streams=1, length=400)),
                                    (3, dict(streams=1)), (4, dict(streams=1, size=64)), (5, dict(streams=1, size=32))])
def test_state_footprint_within_bound_and_independent_of_height(cfg, kw):
    wl = wl_mod.make(cfg, **kw)
    net = idf.net_from_workload(wl)
    s = net.query_sizes(4, wl["seg_rows"], 0)
    assert s.state_bytes_per_stream <= bound_bytes(wl)
    assert (s.out_h, s.out_w, s.out_c) == wl_mod.output_shape(wl)
    net.destroy()
    # a sample twice as tall (1-D: twice as long) needs exactly the same state
    key = "length" if cfg in (1, 2) else None
    if key:
        wl2 = wl_mod.make(cfg, **dict(kw, length=2 * kw["length"]))
        net2 = idf.net_from_workload(wl2)
        assert net2.query_sizes(4, wl["seg_rows"], 0).state_bytes_per_stream == s.state_bytes_per_stream
        net2.destroy()


# rows a layer has completed that may wait for the next layer's step when a call returns, in the
# staged modes: two rows behind every conv layer (or the pool fused behind it) but the last where
# the matrix-core kernel serves the whole net; in the 1-D cascade, behind every layer but the
# last, the rows one push can complete, as float32
def handover_bytes(wl, staged_2d):
    eb = {"f32": 4, "bf16": 2, "i8": 1}[wl["precision"]]
    h, w = wl["in_h"], wl["in_w"]
    rows = wl["seg_rows"]
    total = 0
    n = len(wl["layers"])
    for i, L in enumerate(wl["layers"]):
        h = wl_mod.out_size(h, L["k_h"], L["s_h"], L["p_h"])
        w = wl_mod.out_size(w, L["k_w"], L["s_w"], L["p_w"])
        if i == n - 1:
            break
        if staged_2d:
            if wl["layers"][i + 1]["kind"] != "maxpool":
                total += 2 * w * L["c_out"] * eb
        else:
            rows = -(-rows // L["s_h"]) if L["s_h"] > 1 else rows      # most rows one push completes
            total += rows * L["c_out"] * 4
    return total


@pytest.mark.parametrize("cfg,staged_2d", [(1, False), (2, False), (3, True), (4, True), (5, True)])
def test_retained_bytes_count_the_rows_waiting_between_layers(cfg, staged_2d, monkeypatch):
    """Everything of a stream that survives from one call to the next: the rolling buffers and held
    rows the paper's bound is about (Sec. 3 last two paragraphs, Fig. 1, Fig. 2), plus, in the
    staged modes, the rows waiting between layers.  Strictly depth-first modes hold only the former."""
    wl = wl_mod.make(cfg, streams=1)
    for var in ("IDF_NO_MFMA", "IDF_NO_ROW_STAGES", "IDF_CASCADE_STAGES"):
        monkeypatch.delenv(var, raising=False)
    net = idf.net_from_workload(wl)
    s = net.query_sizes(8, wl["seg_rows"], 0 if wl["in_h"] else 64)
    assert s.state_bytes_per_stream <= bound_bytes(wl)
    assert s.retained_bytes_per_stream == s.state_bytes_per_stream + s.handover_bytes_per_stream
    assert s.handover_bytes_per_stream == handover_bytes(wl, staged_2d)
    assert s.handover_bytes_per_stream <= s.transit_bytes_per_stream
    monkeypatch.setenv("IDF_NO_ROW_STAGES", "1")
    monkeypatch.setenv("IDF_CASCADE_STAGES", "1")
    t = net.query_sizes(8, wl["seg_rows"], 0 if wl["in_h"] else 64)
    assert t.handover_bytes_per_stream == 0
    assert t.retained_bytes_per_stream == t.state_bytes_per_stream == s.state_bytes_per_stream <= bound_bytes(wl)
    net.destroy()


def test_full_size_state_figures():
    # per-stream retained state of the five full-size configurations never exceeds
    # K_h rows per conv layer + one row per pool
    expect = {1: 288, 2: 11520, 3: 53248}
    for cfg, want in expect.items():
        kw = dict(streams=1)
        wl = wl_mod.make(cfg, **kw)
        net = idf.net_from_workload(wl)
        s = net.query_sizes(1, wl["seg_rows"], 0)
        assert s.state_bytes_per_stream <= want
        net.destroy()


def test_query_sizes_errors():
    wl = wl_mod.make(1, streams=1, length=64)
    net = idf.net_from_workload(wl)
    with pytest.raises(idf.IdfError):
        net.query_sizes(0, 1, 0)
    net.destroy()
    un = idf.Net("f32", 0, 1, 1, [conv(1, 4, 3, 1)], [np.zeros((4, 1, 3, 1), np.float32)])
    with pytest.raises(idf.IdfError):
        un.query_sizes(1, 4, 0)          # unbounded needs an explicit output capacity
    assert un.query_sizes(1, 4, 64).out_h == 0
    un.destroy()


def test_eager_workspace_size_and_refusals():
    import ctypes as C
    L = idf.load_library()
    nb = C.c_size_t()
    # a net with a bias keeps every level whole: announced value and delta per level (input + 5
    # layers), state for the 4 conv layers, 4 bytes each
    wl = wl_mod.make(3, streams=2, size=8, channels=(4, 4, 4, 4))
    wl["biases"][0] = np.zeros(4, dtype=np.float32)
    net = idf.net_from_workload(wl)
    assert L.idf_query_eager_bytes(net._h, 2, 1, C.byref(nb)) == 0
    maps = [8 * 8 * 3, 8 * 8 * 4, 8 * 8 * 4, 4 * 4 * 4, 4 * 4 * 4, 4 * 4 * 4]
    least = 2 * 4 * (2 * sum(maps) + maps[1] + maps[2] + maps[4] + maps[5])
    assert least <= nb.value <= least + 20 * 256
    net.destroy()
    wl1 = wl_mod.make(2, streams=1, length=200, channels=(4, 4, 4, 4, 4, 4))
    net1 = idf.Net("f32", 0, 1, 1, wl1["layers"], wl1["weights"])       # unbounded: no output map to keep
    assert L.idf_query_eager_bytes(net1._h, 1, 1, C.byref(nb)) == binding.IDF_EUNSUPPORTED
    net1.destroy()


def test_eager_rings_do_not_grow_with_the_sample_height():
    """Without biases eager emission keeps per level only the cone of rows a later segment can still
    reach (Sec. 3: a single input component reaches a patch that widens by K-1 per layer; Sec. 3
    last paragraph, Fig. 2: a row of cones for 2-D input): everything but the output map, which is
    kept whole, is independent of the height and grows with the rows pushed at once."""
    import ctypes as C
    L = idf.load_library()

    def need(size_h, seg):
        wl = wl_mod.make(3, streams=1, size=16, channels=(4, 4, 4, 4))
        # same net on a taller sample: only in_h differs
        net = idf.Net("f32", size_h, 16, 3, wl["layers"], wl["weights"], wl["biases"])
        nb = C.c_size_t()
        assert L.idf_query_eager_bytes(net._h, 1, seg, C.byref(nb)) == 0
        out_map = (size_h // 2) * 8 * 4 * 4                     # last level's announced values, kept whole
        net.destroy()
        return nb.value, out_map
    a, oa = need(32, 1)
    b, ob = need(64, 1)
    c, oc = need(64, 4)
    assert abs((b - ob) - (a - oa)) <= 16 * 256                 # (alignment of the pieces aside)
    assert c > b
    # rows kept at depth n of 3 x 3 layers: 1 + 2 n cone rows (one push of one row), halved by the pool
    # level: 0 input, 1 conv, 2 conv, 3 pool, 4 conv, 5 conv
    cone = [1, 3, 5, 3, 5, 7]
    row = [16 * 3, 16 * 4, 16 * 4, 8 * 4, 8 * 4, 8 * 4]
    # announced + delta per level, state for conv levels; level 2 keeps one more row for the pool's window
    least = sum(4 * r * k * (3 if lv in (1, 2, 4, 5) else 2) for lv, (r, k) in enumerate(zip(row, cone))) - 4 * row[5] * cone[5]
    assert least <= a - oa <= 2 * least + 16 * 256


def test_volume_net_description_and_sizes():
    """idf_create_net_volume on the host: validation, output shape, and the state of k_d slabs per layer."""
    from paper_1804_10727_amd.binding import VolumeNet
    L = [dict(c_in=2, c_out=4, k=(3, 3, 3), s=(1, 1, 1), p=(1, 1, 1), act="relu"),
         dict(c_in=4, c_out=6, k=(2, 3, 3), s=(1, 2, 2), p=(0, 1, 1), act="relu")]
    w = [np.zeros((4, 2, 3, 3, 3), np.float32), np.zeros((6, 4, 2, 3, 3), np.float32)]
    net = VolumeNet("f32", 9, 10, 8, 2, L, w)
    sz = net.query_sizes(2)
    # slabs 9 -> 9 -> 8; rows 10 -> 10 -> 5; columns 8 -> 8 -> 4, folded into the channels with c_out
    assert (int(sz.out_h), sz.out_w, sz.out_c) == (8, 5, 4 * 6)
    # k_d slabs of c per layer, 4 bytes a cell: 3 x (10 x 8 x 4) + 2 x (5 x 4 x 6)
    assert sz.state_bytes_per_stream == (3 * 10 * 8 * 4 + 2 * 5 * 4 * 6) * 4
    net.destroy()
    with pytest.raises(idf.IdfError) as e:                  # channel chain
        VolumeNet("f32", 9, 10, 8, 3, L, w)
    assert e.value.code == binding.IDF_EINVAL
    with pytest.raises(idf.IdfError) as e:                  # window wider than the volume along the column axis
        VolumeNet("f32", 9, 10, 2, 2, [dict(L[0], p=(1, 1, 0))], w[:1])
    assert e.value.code == binding.IDF_EINVAL
    with pytest.raises(idf.IdfError) as e:                  # no slabs per sample given
        VolumeNet("f32", 0, 10, 8, 2, L, w)
    assert e.value.code == binding.IDF_EINVAL
    with pytest.raises(idf.IdfError) as e:                  # too wide once the column axis is folded in
        VolumeNet("f32", 9, 10, 4096, 2, [dict(L[0], k=(3, 3, 1), p=(1, 1, 0))], [np.zeros((4, 2, 3, 3, 1), np.float32)])
    assert e.value.code == binding.IDF_EUNSUPPORTED
    with pytest.raises(idf.IdfError):                       # missing weights
        VolumeNet("f32", 9, 10, 8, 2, L, [w[0], None])
