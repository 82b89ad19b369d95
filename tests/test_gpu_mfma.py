"""GPU parity for the matrix-core conv path on shapes the five configurations do not reach: odd
widths and heights (ragged tiles, pools that drop a row/column), output channels that fill
only part of a tile, several rows per push, streams out of step, bias."""
import numpy as np
import pytest

import workloads as wl_mod
from workloads import conv, maxpool, round_to_bf16
from helpers import check_stream, gpu_run, oracle_stream

pytestmark = pytest.mark.gpu


def bf16_net(H, W, streams, seed, with_bias=False):
    rng = np.random.default_rng(seed)
    layers = [conv(3, 16, 3, 3, p_h=1, p_w=1), conv(16, 32, 3, 3, p_h=1, p_w=1), maxpool(32),
              conv(32, 80, 3, 3, p_h=1, p_w=1), maxpool(80), conv(80, 64, 3, 3, p_h=1, p_w=1)]
    x = rng.random((streams, H, W, 3), dtype=np.float32)
    x[rng.random((streams, H, W)) < 0.4] = 0
    # one stream with a long empty stretch: whole K-steps without events
    x[0, :, W // 3:] = 0
    ws = [None if L["kind"] != "conv" else
          round_to_bf16(rng.normal(0, np.sqrt(2.0 / (L["c_in"] * 9)), size=(L["c_out"], L["c_in"], 3, 3)).astype(np.float32))
          for L in layers]
    bs = [None if (L["kind"] != "conv" or not with_bias) else rng.normal(0, 0.1, size=(L["c_out"],)).astype(np.float32)
          for L in layers]
    return dict(name="bf16_odd", precision="bf16", in_h=H, in_w=W, in_c=3, layers=layers, weights=ws, biases=bs,
                x=round_to_bf16(x), seg_rows=1, streams=streams)


def i8_net(H, W, streams, seed):
    rng = np.random.default_rng(seed)
    q = dict(act="relu_shr_clamp", shr=4, clamp_hi=15)
    layers = [conv(1, 16, 3, 3, p_h=1, p_w=1, **q), conv(16, 16, 3, 3, p_h=1, p_w=1, **q), maxpool(16),
              conv(16, 32, 3, 3, p_h=1, p_w=1, **q), maxpool(32), conv(32, 48, 3, 3, p_h=1, p_w=1, **q),
              conv(48, 64, 3, 3, p_h=1, p_w=1, act="relu")]
    x = rng.integers(0, 16, size=(streams, H, W, 1)).astype(np.int8)
    x[rng.random((streams, H, W)) < 0.7] = 0
    x[0, :, : W // 2] = 0
    ws = [None if L["kind"] != "conv" else rng.integers(-8, 8, size=(L["c_out"], L["c_in"], 3, 3)).astype(np.int8)
          for L in layers]
    bs = [None if L["kind"] != "conv" else rng.integers(-20, 20, size=(L["c_out"],)).astype(np.int32) for L in layers]
    return dict(name="i8_odd", precision="i8", in_h=H, in_w=W, in_c=1, layers=layers, weights=ws, biases=bs,
                x=x, seg_rows=1, streams=streams)


def _all_mfma(st, W):
    kinds = st.layer_kernels()
    if W >= 8:          # narrower inputs shrink to width 1, which the generic kernel serves
        assert all(k == "conv3x3_mfma" for k in kinds), kinds
    else:
        assert kinds[0] == "conv3x3_mfma"


@pytest.mark.parametrize("H,W,seg", [(21, 37, 1), (21, 37, 4), (34, 70, 1), (12, 131, 3), (9, 5, 1)])
def test_bf16_odd_shapes(H, W, seg):
    wl = bf16_net(H, W, 3, seed=H * 100 + W, with_bias=(seg != 1))
    out, st, net = gpu_run(wl, seg_rows=seg, return_streams=True)
    _all_mfma(st, W)
    for b in range(wl["streams"]):
        check_stream(wl, out[b], b)
    # the first layer sees the same events as the oracle: its counters are exact
    _, e_st = oracle_stream(wl, 0, emit_round="bf16")
    g = st.get_stats(0)
    assert g["events_in"][0] == e_st["events_in"][0] and g["macs"][0] == e_st["macs"][0]
    assert np.allclose(g["events_in"].astype(float), e_st["events_in"].astype(float), rtol=5e-3)
    st.close(); net.destroy()


@pytest.mark.parametrize("H,W,seg", [(30, 50, 1), (30, 50, 3), (17, 67, 1), (8, 140, 8), (5, 4, 1)])
def test_int8_odd_shapes_bit_exact(H, W, seg):
    wl = i8_net(H, W, 3, seed=H * 100 + W)
    out, st, net = gpu_run(wl, seg_rows=seg, return_streams=True)
    _all_mfma(st, W)
    for b in range(wl["streams"]):
        check_stream(wl, out[b], b)
        _, e_st = oracle_stream(wl, b)
        g = st.get_stats(b)
        assert g["events_in"].tolist() == e_st["events_in"].tolist()
        assert g["macs"].tolist() == e_st["macs"].tolist()
    st.close(); net.destroy()


def test_streams_out_of_step_on_the_matrix_core_path():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = i8_net(16, 40, 5, seed=7)
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 5, max_seg_rows=2)
    x = input_tensor(wl)
    order = np.array([3, 0], dtype=np.int32)
    st.push_segment(x[[3, 0], 0:2].contiguous(), stream_ids=order)       # two streams run ahead
    H = 16
    # everybody else catches up one row at a time, then all finish together two rows at a time
    for r in range(2):
        ids = np.array([1, 2, 4], dtype=np.int32)
        st.push_segment(x[[1, 2, 4], r:r + 1].contiguous(), stream_ids=ids)
    for r in range(2, H, 2):
        st.push_segment(x[:, r:r + 2].contiguous())
    out, first, cnt = st.read_outputs(int(st.sizes.out_h))
    torch.cuda.synchronize()
    assert (cnt == st.sizes.out_h).all()
    o = out.cpu().numpy()
    for b in range(5):
        check_stream(wl, o[b], b)
    st.close(); net.destroy()


def _piecewise(wl, seg, reads_after, env=None):
    """Whole sample seg rows per push, reading after the pushes listed; returns rows per stream."""
    import os
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    saved = {k: os.environ.get(k) for k in (env or {})}
    os.environ.update(env or {})
    try:
        net = idf.net_from_workload(wl)
        st = idf.Streams(net, wl["streams"], max_seg_rows=seg)
    finally:
        for k, v in saved.items():
            if v is None:
                del os.environ[k]
            else:
                os.environ[k] = v
    x = input_tensor(wl)
    B, H = wl["streams"], wl["in_h"]
    got = [[] for _ in range(B)]

    def read(max_rows):
        out, first, cnt = st.read_outputs(max_rows)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        for b in range(B):
            if cnt[b]:
                assert first[b] == sum(len(c) for c in got[b])
                got[b].append(o[b, :cnt[b]].copy())
    for i, r in enumerate(range(0, H, seg)):
        st.push_segment(x[:, r:r + seg].contiguous())
        if i in reads_after:
            read(3)
    for _ in range(int(st.sizes.out_h) // 3 + 2):
        read(3)
    stats = [st.get_stats(b) for b in range(B)]
    st.close(); net.destroy()
    return [np.concatenate(g) for g in got], stats


@pytest.mark.parametrize("seg", [1, 3])
def test_rows_between_layers_never_show(seg):
    """Layers run one launch behind each other across pushes; reads in between, the end of the
    sample (two rows complete at once in every layer) and the counters must not show it."""
    wl = i8_net(26, 44, 3, seed=11)
    n_push = (26 + seg - 1) // seg
    a, sa = _piecewise(wl, seg, reads_after={0, 1, 2, 5, n_push - 2, n_push - 1})
    b, sb = _piecewise(wl, seg, reads_after={4}, env={"IDF_NO_ROW_STAGES": "1"})
    for i in range(3):
        check_stream(wl, a[i], i)
        assert np.array_equal(a[i], b[i])
        assert sa[i]["events_in"].tolist() == sb[i]["events_in"].tolist()
        assert sa[i]["macs"].tolist() == sb[i]["macs"].tolist()
    wl = bf16_net(20, 40, 2, seed=12, with_bias=True)
    a, _ = _piecewise(wl, seg, reads_after={0, 3, 4})
    b, _ = _piecewise(wl, seg, reads_after=set(), env={"IDF_NO_ROW_STAGES": "1"})
    for i in range(2):
        check_stream(wl, a[i], i)
        assert np.array_equal(a[i], b[i])


def test_two_samples_through_the_staged_layers():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = i8_net(18, 36, 4, seed=13)
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 2, max_seg_rows=2)
    x = input_tensor(wl)
    # the second sample starts while rows of the first are still between layers
    for r in range(0, 18, 2):
        st.push_segment(x[0:2, r:r + 2].contiguous())
    out1, _, c1 = st.read_outputs(int(st.sizes.out_h))
    for r in range(0, 18, 2):
        st.push_segment(x[2:4, r:r + 2].contiguous())
    out2, _, c2 = st.read_outputs(int(st.sizes.out_h))
    torch.cuda.synchronize()
    assert (c1 == st.sizes.out_h).all() and (c2 == st.sizes.out_h).all()
    for i in range(2):
        check_stream(wl, out1[i].cpu().numpy(), i)
        check_stream(wl, out2[i].cpu().numpy(), 2 + i)
    st.close(); net.destroy()
