"""GPU parity for the 1-D cascade when its layers are dealt to stages that run side by side,
each one push behind the stage before: what a caller can observe (rows readable after a
read, counters, state after pushes of only some streams) must not depend on that."""
import os

import numpy as np
import pytest

import workloads as wl_mod
from helpers import TOL, check_stream, oracle_dense, oracle_stream, rel_err

pytestmark = pytest.mark.gpu


def _run(wl, seg, reads_at, stages=None, ids_plan=None, batch=None):
    """Push the whole sample seg rows at a time, reading after the pushes listed in reads_at.
    batch: hold back up to that many pushes per launch (idf_set_push_batching)."""
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    old = os.environ.get("IDF_CASCADE_STAGES")
    if stages is not None:
        os.environ["IDF_CASCADE_STAGES"] = str(stages)
    try:
        net = idf.net_from_workload(wl)
        st = idf.Streams(net, wl["streams"], max_seg_rows=seg)
    finally:
        if stages is not None:
            if old is None:
                del os.environ["IDF_CASCADE_STAGES"]
            else:
                os.environ["IDF_CASCADE_STAGES"] = old
    assert all(k == "cascade1d" for k in st.layer_kernels())
    x = input_tensor(wl)
    B, H = wl["streams"], wl["in_h"]
    got = [[] for _ in range(B)]
    if batch:
        st.set_push_batching(batch)
    # a held-back segment is read when its launch runs: every segment stays alive until the end
    segs = [x[:, r:r + seg].contiguous() for r in range(0, H, seg)]

    def read():
        out, first, cnt = st.read_outputs(int(st.sizes.out_h))
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        for b in range(B):
            if cnt[b]:
                assert first[b] == sum(len(c) for c in got[b])
                got[b].append(o[b, :cnt[b]].copy())
    for i, r in enumerate(range(0, H, seg)):
        st.push_segment(segs[i])
        if i in reads_at:
            read()
    read()
    stats = [st.get_stats(b) for b in range(B)]
    st.close(); net.destroy()
    return [np.concatenate(g) for g in got], stats


def test_reads_between_pushes_see_every_completed_row():
    wl = wl_mod.make(2, streams=5, length=640, channels=(8, 16, 16, 32, 32, 64))
    n_push = 640 // 16
    outs, stats = _run(wl, 16, reads_at={0, 1, 2, 7, 8, 20, n_push - 2})
    for b in range(5):
        check_stream(wl, outs[b], b)
        _, e_st = oracle_stream(wl, b)
        assert stats[b]["events_in"][0] == e_st["events_in"][0]
        assert np.allclose(stats[b]["events_in"].astype(float), e_st["events_in"].astype(float), rtol=5e-3)


@pytest.mark.parametrize("seg", [1, 5, 16])
def test_staged_and_unstaged_agree_bit_for_bit(seg):
    wl = wl_mod.make(2, streams=3, length=400, channels=(8, 8, 16, 16, 32, 64))
    a, sa = _run(wl, seg, reads_at={3})
    b, sb = _run(wl, seg, reads_at={3}, stages=1)
    c, sc = _run(wl, seg, reads_at=set(), stages=2)
    for i in range(3):
        assert np.array_equal(a[i], b[i]) and np.array_equal(a[i], c[i])
        assert sa[i]["events_in"].tolist() == sb[i]["events_in"].tolist() == sc[i]["events_in"].tolist()
        assert sa[i]["macs"].tolist() == sb[i]["macs"].tolist()


def test_pushes_of_some_streams_between_pushes_of_all():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(2, streams=4, length=320, channels=(8, 8, 8, 16, 16, 16))
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 4, max_seg_rows=16)
    x = input_tensor(wl)
    # all in step, then streams 2 and 0 run ahead (segments of all streams are still between
    # stages at that point), the others catch up, all in step again
    for r in range(0, 96, 16):
        st.push_segment(x[:, r:r + 16].contiguous())
    ahead = np.array([2, 0], dtype=np.int32)
    for r in range(96, 160, 16):
        st.push_segment(x[[2, 0], r:r + 16].contiguous(), stream_ids=ahead)
    behind = np.array([1, 3], dtype=np.int32)
    for r in range(96, 160, 8):
        st.push_segment(x[[1, 3], r:r + 8].contiguous(), stream_ids=behind)
    for r in range(160, 320, 16):
        st.push_segment(x[:, r:r + 16].contiguous())
    out, first, cnt = st.read_outputs(int(st.sizes.out_h))
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    for b in range(4):
        d = oracle_dense(wl, b)
        assert cnt[b] == d.shape[0]
        assert rel_err(o[b, :cnt[b]], d) <= TOL["f32"]
    st.close(); net.destroy()


def test_single_stream_one_sample_per_push_with_bias():
    wl = wl_mod.make(1, length=300)
    outs, _ = _run(wl, 1, reads_at={0, 1, 2, 3, 10, 11})
    check_stream(wl, outs[0], 0)


def _deep_1d(streams, length, seed=77):
    """Eight conv1d layers (kernel 3, valid, one of them stride 2, biases on two): as many stages
    as the kernel's descriptor table holds."""
    rng = np.random.default_rng(seed)
    x = rng.normal(0.0, 1.0, size=(streams, length, 1, 1)).astype(np.float32)
    x[rng.random(x.shape) < 0.5] = 0.0
    chans = (1, 8, 8, 16, 16, 16, 32, 32, 32)
    layers = [wl_mod.conv(chans[i], chans[i + 1], 3, 1, s=(2 if i == 2 else 1)) for i in range(8)]
    weights = wl_mod._normal_weights(rng, layers, 2.0)
    biases = [None] * 8
    for i in (0, 5):
        biases[i] = rng.normal(0.0, 0.1, size=chans[i + 1]).astype(np.float32)
    return wl_mod._finish("deep_1d_k3", "f32", length, 1, 1, layers, weights, biases, x, 4)


def test_eight_layers_in_eight_stages():
    wl = _deep_1d(4, 200)
    a, sa = _run(wl, 4, reads_at={0, 5, 6, 30})
    b, sb = _run(wl, 4, reads_at={5}, stages=1)
    for i in range(4):
        check_stream(wl, a[i], i)
        assert np.array_equal(a[i], b[i])
        assert sa[i]["events_in"].tolist() == sb[i]["events_in"].tolist()
        assert sa[i]["macs"].tolist() == sb[i]["macs"].tolist()


@pytest.mark.parametrize("streams", [130, 131])
def test_more_streams_than_a_stage_per_layer_allows(streams):
    # 2 x 256 workgroups fit at once: three stages for 130 streams (filled up to four for the XCD
    # mapping when the stream count is even, not when it is odd)
    wl = wl_mod.make(2, streams=streams, length=160, channels=(8, 8, 16, 16, 16, 16))
    a, _ = _run(wl, 16, reads_at={2})
    b, _ = _run(wl, 16, reads_at=set(), stages=1)
    for i in (0, 1, 64, streams - 2, streams - 1):
        check_stream(wl, a[i], i)
    for i in range(streams):
        assert np.array_equal(a[i], b[i])


def test_reset_mid_flight_on_unbounded_streams():
    """Unbounded 1-D streams (no sample length: they never flush), a small output ring read piece by
    piece; one stream is reset while segments of all streams are still between the stages, starts a
    new signal at row 0 and runs on beside the others, which must not notice."""
    import torch
    import paper_1804_10727_amd as idf
    wl = wl_mod.make(2, streams=3, length=640, channels=(8, 8, 16, 16, 16, 16))
    layers, ws = wl["layers"], wl["weights"]
    net = idf.Net("f32", 0, 1, 1, layers, ws)                      # in_h = 0: unbounded
    st = idf.Streams(net, 3, max_seg_rows=16, out_cap_rows=24)
    assert st.sizes.out_h == 0
    x = torch.from_numpy(wl["x"]).to("cuda:0")                     # [3][640][1][1]
    second = torch.from_numpy(wl_mod.make(2, streams=1, length=640, channels=(8, 8, 16, 16, 16, 16), seed=5)["x"]).to("cuda:0")
    got = [[], [], []]
    new1 = []

    def read_all():
        for _ in range(3):
            out, first, cnt = st.read_outputs(16)
            o = out.cpu().numpy()
            for b in range(3):
                (got[b] if (b != 1 or not new1_started[0]) else new1).append(o[b, :cnt[b]])

    new1_started = [False]
    pos1 = 0
    for i, r in enumerate(range(0, 640, 16)):
        if i == 9:
            # segments 6..8 of all streams are still on their way through the stages
            read_all()
            st.reset(stream_ids=[1])
            new1_started[0] = True
        if new1_started[0]:
            seg = torch.cat([x[[0], r:r + 16], second[[0], pos1:pos1 + 16], x[[2], r:r + 16]]).contiguous()
            pos1 += 16
        else:
            seg = x[:, r:r + 16].contiguous()
        st.push_segment(seg)
        if i % 2 == 1:
            read_all()
    read_all()
    torch.cuda.synchronize()
    import oracle
    for b, sig in ((0, wl["x"][0]), (2, wl["x"][2])):
        want = oracle.dense(layers, sig, ws, None)
        g = np.concatenate(got[b])
        assert g.shape == want.shape
        assert rel_err(g, want) <= TOL["f32"], b
    want_old = oracle.dense(layers, wl["x"][1][:9 * 16], ws, None)       # what stream 1 had completed before the reset
    g_old = np.concatenate(got[1])
    assert g_old.shape == want_old.shape and rel_err(g_old, want_old) <= TOL["f32"]
    want_new = oracle.dense(layers, second.cpu().numpy()[0][:pos1], ws, None)
    g_new = np.concatenate(new1)
    assert g_new.shape == want_new.shape and rel_err(g_new, want_new) <= TOL["f32"]
    st.close(); net.destroy()


def _same_up_to_association(a, b):
    """Two float32 results that add the same products in a different association."""
    return rel_err(a, b.astype(np.float64)) <= 2e-6


@pytest.mark.parametrize("seg,batch", [(16, 8), (5, 3), (1, 8), (1, 16), (16, 2), (4, 16)])
def test_pushes_held_back_and_run_several_per_launch(seg, batch):
    """Throughput mode: up to `batch` pushes in step share one launch; a stage takes consecutive
    segments together while their rows fit one step, the rolling buffers staying in LDS from one
    step to the next.  Outputs are those of one launch per push up to the association of the
    float32 sums (rows of several segments are added in one pass), the counters the same, with
    reads falling between launches and inside a group of held-back pushes, with a number of pushes
    that leaves a remainder, staged and unstaged."""
    wl = wl_mod.make(2, streams=3, length=400, channels=(8, 8, 16, 16, 32, 64))
    n_push = (400 + seg - 1) // seg
    ref, sref = _run(wl, seg, reads_at={3}, stages=1)
    a, sa = _run(wl, seg, reads_at={1, 2, 10, n_push - 2}, batch=batch)
    b, sb = _run(wl, seg, reads_at=set(), batch=batch)
    c, sc = _run(wl, seg, reads_at={4}, stages=1, batch=batch)
    for i in range(3):
        check_stream(wl, a[i], i)
        assert a[i].shape == ref[i].shape
        assert _same_up_to_association(a[i], ref[i]) and _same_up_to_association(b[i], ref[i]) and _same_up_to_association(c[i], ref[i])
        for sx in (sa, sb, sc):
            assert sx[i]["events_in"][0] == sref[i]["events_in"][0]      # the input's events: exact
            assert np.allclose(sx[i]["events_in"].astype(float), sref[i]["events_in"].astype(float), rtol=1e-3)
            assert np.allclose(sx[i]["macs"].astype(float), sref[i]["macs"].astype(float), rtol=1e-3)


def test_held_back_pushes_and_pushes_of_some_streams():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(2, streams=4, length=320, channels=(8, 8, 8, 16, 16, 16))
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 4, max_seg_rows=16)
    st.set_push_batching(4)
    x = input_tensor(wl)
    keep = []

    def push(rows, ids=None):
        keep.append(rows)
        st.push_segment(rows, stream_ids=ids)
    for r in range(0, 96, 16):                    # six pushes in step: one full group, two held back
        push(x[:, r:r + 16].contiguous())
    ahead = np.array([2, 0], dtype=np.int32)      # a push of two streams: what is held back runs first
    for r in range(96, 160, 16):
        push(x[[2, 0], r:r + 16].contiguous(), ahead)
    behind = np.array([1, 3], dtype=np.int32)
    for r in range(96, 160, 8):
        push(x[[1, 3], r:r + 8].contiguous(), behind)
    for r in range(160, 320, 16):
        push(x[:, r:r + 16].contiguous())
    out, first, cnt = st.read_outputs(int(st.sizes.out_h))
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    for b in range(4):
        d = oracle_dense(wl, b)
        assert cnt[b] == d.shape[0]
        assert rel_err(o[b, :cnt[b]], d) <= TOL["f32"]
    with pytest.raises(idf.IdfError):
        st.set_push_batching(17)
    st.close(); net.destroy()


def test_single_stream_one_sample_per_push_held_back():
    wl = wl_mod.make(1, length=300)
    ref, _ = _run(wl, 1, reads_at=set(), stages=1)
    outs, _ = _run(wl, 1, reads_at={0, 1, 2, 3, 10, 11, 100}, batch=16)
    check_stream(wl, outs[0], 0)
    assert _same_up_to_association(outs[0], ref[0])
