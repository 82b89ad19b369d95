"""GPU test of snapshot / restore of a stream's retained state (the hidden state of the recurrent
view, Sec. 5): a stream stopped half way, its state parked in a caller's buffer, resumed in another
stream slot, must deliver exactly what an uninterrupted stream delivers."""
import numpy as np
import pytest

import workloads as wl_mod
from helpers import check_stream

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,kw,seg,cut", [
    (2, dict(streams=3, length=320, channels=(8, 8, 16, 16, 32, 32)), 16, 9),
    (4, dict(streams=3, size=24, channels=(4, 4, 8, 8, 16, 16, 16, 16)), 1, 13),
    (3, dict(streams=3, size=16, channels=(8, 8, 16, 16)), 2, 3),
])
def test_resume_in_another_stream(cfg, kw, seg, cut):
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(cfg, **kw)
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 3, max_seg_rows=seg)
    st.enable_head()
    x = input_tensor(wl)
    H = wl["in_h"]
    out_h = int(st.sizes.out_h) if st.sizes.out_h > 0 else 10 ** 6
    n_push = H // seg
    # stream 1 receives the first `cut` segments of sample 1 (the others stay idle)
    one = np.array([1], dtype=np.int32)
    for i in range(cut):
        st.push_segment(x[[1], i * seg:(i + 1) * seg].contiguous(), stream_ids=one)
    if cfg == 2:
        with pytest.raises(idf.IdfError):
            st.snapshot(1)                               # completed rows not read yet
    out, first, cnt = st.read_outputs(min(out_h, 4096), stream_ids=one)
    head = out[0, :cnt[0]].cpu().numpy()
    buf, pos = st.snapshot(1)
    assert pos[0] == (cut * seg) % H and pos[1] == cnt[0]
    stats_before = st.get_stats(1)
    # the slot is reused for something else, the state comes back in slot 2
    st.reset(stream_ids=[1])
    st.push_segment(x[[0], 0:seg].contiguous(), stream_ids=one)
    st.restore(2, buf, pos)
    two = np.array([2], dtype=np.int32)
    for i in range(cut, n_push):
        st.push_segment(x[[1], i * seg:(i + 1) * seg].contiguous(), stream_ids=two)
    out, first, cnt2 = st.read_outputs(min(out_h, 4096), stream_ids=two)
    torch.cuda.synchronize()
    assert first[0] == (cnt[0] if st.sizes.out_h > 0 else pos[1])
    tail = out[0, :cnt2[0]].cpu().numpy()
    check_stream(wl, np.concatenate([head, tail]), 1)
    after = st.get_stats(2)
    assert (after["events_in"] >= stats_before["events_in"]).all() and after["events_in"][0] > stats_before["events_in"][0]
    rows, mean = st.read_head(stream_ids=two)
    full = np.concatenate([head, tail]).astype(np.float64)
    assert rows[0] == full.shape[0]
    ref = full.reshape(-1, full.shape[-1]).mean(axis=0)
    assert np.max(np.abs(mean[0] - ref)) <= 1e-5 * max(np.max(np.abs(ref)), 1e-30)
    st.close(); net.destroy()
