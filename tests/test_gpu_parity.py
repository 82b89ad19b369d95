"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

import workloads as wl_mod
from workloads import conv, maxpool
from helpers import (TOL, check_stream, gpu_run, oracle_dense, oracle_many, oracle_stream, rel_err)

pytestmark = pytest.mark.gpu

SMALL = {
    1: dict(streams=3, length=301),
    2: dict(streams=5, length=1003, channels=(8, 8, 16, 16, 24, 16)),
    3: dict(streams=7, size=16, channels=(8, 8, 16, 16)),
    4: dict(streams=3, size=40, channels=(4, 4, 8, 8, 16, 16, 16, 16)),
    5: dict(streams=2, size=24, channels=(8, 8, 16, 16, 32, 32, 32)),
}
# several tiles and a ragged tail for the kernels, still seconds for the oracle
MEDIUM = {
    2: dict(streams=3, length=2100),
    3: dict(streams=9, size=32),
    4: dict(streams=2, size=100),
    5: dict(streams=2, size=52, channels=(64, 64, 128, 128, 256, 256, 256)),
}


def _stats_match(wl, st, b, exact):
    e_out, e_st = oracle_stream(wl, b, emit_round=("bf16" if wl["precision"] == "bf16" else None))
    g = st.get_stats(b)
    if exact:
        assert g["events_in"].tolist() == e_st["events_in"].tolist()
        assert g["macs"].tolist() == e_st["macs"].tolist()
    else:
        # first layer sees the same input: exact; deeper layers may differ where a sum rounds to
        # the other side of zero
        assert g["events_in"][0] == e_st["events_in"][0] and g["macs"][0] == e_st["macs"][0]
        assert np.allclose(g["events_in"].astype(float), e_st["events_in"].astype(float), rtol=2e-3)
        assert np.allclose(g["macs"].astype(float), e_st["macs"].astype(float), rtol=2e-3)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_small_configs_all_streams(cfg):
    wl = wl_mod.make(cfg, **SMALL[cfg])
    out, st, net = gpu_run(wl, return_streams=True)
    for b in range(wl["streams"]):
        check_stream(wl, out[b], b)
    _stats_match(wl, st, 0, exact=(wl["precision"] == "i8"))
    _stats_match(wl, st, wl["streams"] - 1, exact=(wl["precision"] == "i8"))
    # retained state within K_h rows per conv layer + one row per pool
    sb = st.get_stats(0)["state_bytes"]
    eb = {"f32": 4, "bf16": 2, "i8": 1}[wl["precision"]]
    shapes = [(0, wl["in_w"], wl["in_c"])]
    for L, s_b in zip(wl["layers"], sb):
        w_in = shapes[-1][1]
        w_o = wl_mod.out_size(w_in, L["k_w"], L["s_w"], L["p_w"])
        shapes.append((0, w_o, L["c_out"]))
        bound = L["k_h"] * w_o * L["c_out"] * 4 if L["kind"] == "conv" else w_in * L["c_out"] * eb
        assert s_b <= bound
    st.close(); net.destroy()


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_medium_configs(cfg):
    wl = wl_mod.make(cfg, **MEDIUM[cfg])
    out = gpu_run(wl)
    for b in range(wl["streams"]):
        check_stream(wl, out[b], b)


@pytest.mark.parametrize("seg", [1, 2, 5, 16, 37])
def test_segment_length_does_not_matter_1d(seg):
    wl = wl_mod.make(2, streams=2, length=500, channels=(8, 8, 8, 8, 8, 8))
    out = gpu_run(wl, seg_rows=seg)
    for b in range(2):
        check_stream(wl, out[b], b)


@pytest.mark.parametrize("seg", [2, 3, 7, 24])
def test_several_rows_per_push_2d(seg):
    wl = wl_mod.make(3, streams=2, size=24, channels=(8, 8, 8, 8))
    out = gpu_run(wl, seg_rows=seg)
    for b in range(2):
        check_stream(wl, out[b], b)
    wl4 = wl_mod.make(4, streams=1, size=24, channels=(4, 4, 4, 4, 8, 8, 8, 8))
    out = gpu_run(wl4, seg_rows=seg)
    check_stream(wl4, out[0], 0)


def test_odd_shapes_strides_bias_pool():
    """A net unlike the five configs: odd sizes, strides in both directions, asymmetric kernels,
    channel counts that are not multiples of anything, biases, identity activation, pools."""
    rng = np.random.default_rng(42)
    layers = [conv(3, 5, 3, 3, p_h=1, p_w=1), conv(5, 7, 5, 3, s=2, p_h=2, p_w=1), maxpool(7),
              conv(7, 70, 3, 3, p_h=1, p_w=0, act="none"), conv(70, 3, 1, 1)]
    H, W = 37, 45
    x = rng.normal(size=(4, H, W, 3)).astype(np.float32)
    x[rng.random((4, H, W)) < 0.5] = 0
    ws = [None if L["kind"] != "conv" else
          (rng.normal(size=(L["c_out"], L["c_in"], L["k_h"], L["k_w"])) / np.sqrt(L["c_in"] * L["k_h"] * L["k_w"])).astype(np.float32)
          for L in layers]
    bs = [None if L["kind"] != "conv" else rng.normal(size=(L["c_out"],)).astype(np.float32) * 0.2 for L in layers]
    wl = dict(name="odd", precision="f32", in_h=H, in_w=W, in_c=3, layers=layers, weights=ws, biases=bs,
              x=x, seg_rows=1, streams=4)
    for seg in (1, 4):
        out = gpu_run(wl, seg_rows=seg)
        for b in range(4):
            check_stream(wl, out[b], b)


def test_zero_input_costs_nothing():
    for cfg in (2, 3, 4, 5):
        wl = wl_mod.make(cfg, **SMALL[cfg])
        wl["x"][:] = 0
        out, st, net = gpu_run(wl, return_streams=True)
        assert not out.any()
        s = st.get_stats(0)
        assert s["events_in"].sum() == 0 and s["macs"].sum() == 0
        st.close(); net.destroy()


def test_streams_out_of_step_reset_and_piecewise_reads():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(3, streams=6, size=12, channels=(8, 8, 8, 8))
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 6)
    x = input_tensor(wl)
    H = 12
    # streams 4,1 run ahead by 3 rows, in an id order that is neither sorted nor contiguous
    ids = np.array([4, 1], dtype=np.int32)
    for r in range(3):
        st.push_segment(x[[4, 1], r:r + 1].contiguous(), stream_ids=ids)
    assert st.rows_pushed(4) == 3 and st.rows_pushed(0) == 0
    # stream 5 gets garbage and is reset
    st.push_segment(x[[2], 5:6].contiguous(), stream_ids=np.array([5], dtype=np.int32))
    st.reset(stream_ids=[5])
    got = {b: [] for b in range(6)}

    def drain(max_rows=2):
        out, first, cnt = st.read_outputs(max_rows)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        for b in range(6):
            if cnt[b]:
                assert first[b] == sum(len(c) for c in got[b])
                got[b].append(o[b, :cnt[b]].copy())
    for step in range(H):
        rows, idl = [], []
        for b in range(6):
            r = st.rows_pushed(b)
            if b in (4, 1) and step >= H - 3:
                continue
            rows.append(x[b, r:r + 1]); idl.append(b)
        st.push_segment(torch.stack(rows).contiguous(), stream_ids=np.array(idl, dtype=np.int32))
        drain()
    for _ in range(4):
        drain()
    for b in range(6):
        g = np.concatenate(got[b])
        assert g.shape[0] == st.sizes.out_h
        check_stream(wl, g, b)
    # errors: nothing is enqueued, state unchanged
    with pytest.raises(idf.IdfError) as e:
        st.push_segment(x[[0, 0], 0:1].contiguous(), stream_ids=np.array([0, 0], dtype=np.int32))
    assert e.value.code == idf.binding.IDF_EINVAL
    with pytest.raises(idf.IdfError):
        st.push_segment(x[[0], 0:1].contiguous(), stream_ids=np.array([6], dtype=np.int32))
    with pytest.raises(idf.IdfError):
        st.push_segment(x[:, 0:2].contiguous())            # more rows than max_seg_rows
    # second sample straight after the first, without reading in between -> output area full
    for r in range(H - 1):
        st.push_segment(x[:, r:r + 1].contiguous())
    st.read_outputs(64)
    st.push_segment(x[:, H - 1:H].contiguous())
    with pytest.raises(idf.IdfError) as e:
        for r in range(H):
            st.push_segment(x[:, r:r + 1].contiguous())
    assert e.value.code == idf.binding.IDF_ESTATE
    st.close(); net.destroy()


def test_two_samples_back_to_back():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(4, streams=4, size=40, channels=(4, 4, 8, 8, 16, 16, 16, 16))
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 2)
    x = input_tensor(wl)
    for sample in range(2):
        for r in range(40):
            st.push_segment(x[2 * sample:2 * sample + 2, r:r + 1].contiguous())
        out, first, cnt = st.read_outputs(int(st.sizes.out_h))
        torch.cuda.synchronize()
        for i in range(2):
            check_stream(wl, out[i].cpu().numpy(), 2 * sample + i)
    st.close(); net.destroy()


def test_unbounded_1d_stream_with_small_output_ring():
    import torch
    import paper_1804_10727_amd as idf
    wl = wl_mod.make(2, streams=2, length=900, channels=(8, 8, 8, 8, 8, 8))
    net = idf.Net("f32", 0, 1, 1, wl["layers"], wl["weights"])
    st = idf.Streams(net, 2, max_seg_rows=16, out_cap_rows=10)
    x = torch.from_numpy(wl["x"]).cuda()
    chunks = [[], []]
    for r in range(0, 900, 16):
        seg = x[:, r:r + 16].contiguous()
        st.push_segment(seg)
        out, first, cnt = st.read_outputs(10)
        torch.cuda.synchronize()
        for b in range(2):
            if cnt[b]:
                assert first[b] == sum(len(c) for c in chunks[b])
                chunks[b].append(out[b, :cnt[b]].cpu().numpy())
    for b in range(2):
        g = np.concatenate(chunks[b])
        d = oracle_dense(wl, b)
        n = g.shape[0]
        # an unbounded stream never learns that the signal ended: it has every row the 900
        # samples complete, which is all of them for valid padding
        assert n == d.shape[0]
        assert rel_err(g, d) <= TOL["f32"]
    st.close(); net.destroy()


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_generic_kernels_when_the_matrix_core_path_is_off(cfg, monkeypatch):
    """The any-shape kernels serve what the fast kernels do not; with the matrix-core path
    switched off they must carry the 2-D configurations on their own."""
    monkeypatch.setenv("IDF_NO_MFMA", "1")
    kw = {3: dict(streams=3, size=12, channels=(8, 8, 16, 16)),
          4: dict(streams=2, size=24, channels=(4, 4, 8, 8, 16, 16, 16, 16)),
          5: dict(streams=2, size=16, channels=(8, 8, 16, 16, 16, 16, 16))}[cfg]
    wl = wl_mod.make(cfg, **kw)
    out, st, net = gpu_run(wl, return_streams=True)
    assert all(k in ("conv_generic", "pool_generic") for k in st.layer_kernels())
    for b in range(wl["streams"]):
        check_stream(wl, out[b], b)
    st.close(); net.destroy()
