"""GPU parity for pixel segments (Sec. 3: input segments may be arbitrarily small, down to single
components): rows presented a few columns at a time must give what whole rows give."""
import numpy as np
import pytest

import workloads as wl_mod
from helpers import check_stream

pytestmark = pytest.mark.gpu


def _run_in_pixel_segments(wl, seed, streams_subset=None):
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    rng = np.random.default_rng(seed)
    B, H, W = wl["streams"], wl["in_h"], wl["in_w"]
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, B)
    x = input_tensor(wl)
    for r in range(H):
        mode = rng.integers(0, 4)
        if mode == 0:                       # the whole row at once
            st.push_segment(x[:, r:r + 1].contiguous())
            continue
        cuts = [0, W] if mode == 1 else sorted(set([0, W] + rng.integers(1, W, size=int(rng.integers(1, 6))).tolist()))
        if mode == 1:                       # single pixels for part of the row, then the rest
            k = int(rng.integers(1, min(W, 5)))
            cuts = list(range(0, k + 1)) + [W]
        for a, b in zip(cuts[:-1], cuts[1:]):
            st.push_pixels(x[:, r, a:b].contiguous(), a)
    out, first, cnt = st.read_outputs(int(st.sizes.out_h))
    torch.cuda.synchronize()
    assert (cnt == st.sizes.out_h).all()
    o = out.cpu().numpy()
    for b in range(B):
        check_stream(wl, o[b], b)
    stats = [st.get_stats(b) for b in range(B)]
    st.close(); net.destroy()
    return o, stats


def test_int8_rows_in_pixel_segments_bit_exact():
    wl = wl_mod.make(4, streams=3, size=40, channels=(16, 16, 16, 16, 32, 32, 32, 32))
    o, stats = _run_in_pixel_segments(wl, seed=1)
    # the counters see every event exactly once however the row was cut
    import oracle
    for b in range(3):
        _, e_st = oracle.stream_run(wl["layers"], wl["x"][b], wl["weights"], wl["biases"], seg_rows=1, integer=True)
        assert stats[b]["events_in"].tolist() == e_st["events_in"].tolist()
        assert stats[b]["macs"].tolist() == e_st["macs"].tolist()


def test_float_and_bf16_rows_in_pixel_segments():
    _run_in_pixel_segments(wl_mod.make(3, streams=4, size=20, channels=(16, 16, 32, 32)), seed=2)
    _run_in_pixel_segments(wl_mod.make(5, streams=2, size=24, channels=(16, 16, 16, 16, 32, 32, 32)), seed=3)
    # wide rows: several tiles, segments in the middle touch only some of them
    wl = wl_mod.make(4, streams=2, size=136, channels=(16, 16, 16, 16, 16, 16, 16, 16))
    _run_in_pixel_segments(wl, seed=4)


def test_first_layers_the_matrix_core_kernel_does_not_serve(monkeypatch):
    """Pixel segments into a first layer on the generic kernel: every layer on it (the matrix-core kernels
    switched off), and first layers of other shapes -- 5x5 with stride 2 and no padding, 3x3 with stride 2
    and same padding, a 1x3 kernel -- in front of layers the matrix-core kernel takes."""
    from workloads import conv, maxpool
    monkeypatch.setenv("IDF_NO_MFMA", "1")
    _run_in_pixel_segments(wl_mod.make(4, streams=3, size=24, channels=(16, 16, 16, 16, 32, 32, 32, 32)), seed=5)
    _run_in_pixel_segments(wl_mod.make(3, streams=2, size=20, channels=(16, 16, 32, 32)), seed=6)
    monkeypatch.delenv("IDF_NO_MFMA")
    rng = np.random.default_rng(11)
    q = dict(act="relu_shr_clamp", shr=4, clamp_hi=15)
    for first, hw in ((conv(2, 16, 5, 5, s=2, **q), (31, 29)), (conv(2, 16, 3, 3, s=2, p_h=1, p_w=1, **q), (30, 27)),
                      (conv(2, 16, 1, 3, p_w=1, **q), (12, 21))):
        H, W = hw
        layers = [first, conv(16, 16, 3, 3, p_h=1, p_w=1, **q), maxpool(16), conv(16, 32, 3, 3, p_h=1, p_w=1, act="relu")]
        ws = [rng.integers(-8, 8, size=(L["c_out"], L["c_in"], L["k_h"], L["k_w"])).astype(np.int8) if L["kind"] == "conv" else None for L in layers]
        x = (rng.integers(0, 16, size=(2, H, W, 2)) * (rng.random((2, H, W, 2)) < 0.4)).astype(np.int8)
        wl = dict(name="first_layer_shapes", precision="i8", in_h=H, in_w=W, in_c=2, layers=layers, weights=ws,
                  biases=[None] * len(layers), x=x, seg_rows=1, streams=2)
        import oracle
        o, stats = _run_in_pixel_segments(wl, seed=12)
        for b in range(2):
            _, e_st = oracle.stream_run(layers, x[b], ws, wl["biases"], seg_rows=1, integer=True)
            assert stats[b]["events_in"].tolist() == e_st["events_in"].tolist()
            assert stats[b]["macs"].tolist() == e_st["macs"].tolist()


def test_pixel_segment_errors():
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(3, streams=2, size=12, channels=(16, 16, 16, 16))
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 2)
    x = input_tensor(wl)
    st.push_pixels(x[:, 0, 0:5].contiguous(), 0)
    with pytest.raises(idf.IdfError) as e:
        st.push_pixels(x[:, 0, 6:8].contiguous(), 6)            # column 5 is next
    assert e.value.code == idf.binding.IDF_ESTATE
    with pytest.raises(idf.IdfError) as e:
        st.push_segment(x[:, 0:1].contiguous())                 # the row must be finished as pixels
    assert e.value.code == idf.binding.IDF_ESTATE
    with pytest.raises(idf.IdfError) as e:
        st.push_pixels(x[:, 0, 5:12].contiguous()[:, :, :], 6)  # would run past the row
    st.push_pixels(x[:, 0, 5:12].contiguous(), 5)
    assert st.rows_pushed(0) == 1
    st.close(); net.destroy()
    wl1 = wl_mod.make(2, streams=1, length=200, channels=(4, 4, 4, 4, 4, 4))
    net1 = idf.net_from_workload(wl1)
    st1 = idf.Streams(net1, 1, max_seg_rows=16)
    st1.push_pixels(input_tensor(wl1)[:, 0, 0:1].contiguous(), 0)     # a 1-D sample is its own row
    assert st1.rows_pushed(0) == 1
    st1.close(); net1.destroy()
