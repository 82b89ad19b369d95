"""Pushes of several rows on nets served throughout by the matrix-core kernel go through the layers
two rows per launch, the rows between them kept in the accumulators: every value and counter must be
that of one launch per row, bit for bit (the sums are formed in the same order)."""
import os

import numpy as np
import pytest

import workloads as wl_mod
from helpers import check_stream

pytestmark = pytest.mark.gpu


def _run(wl, seg, pairs=True, reads_between=False):
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    if not pairs:
        os.environ["IDF_NO_ROW_PAIRS"] = "1"
    try:
        net = idf.net_from_workload(wl)
        st = idf.Streams(net, wl["streams"], max_seg_rows=max(seg, 2))
    finally:
        os.environ.pop("IDF_NO_ROW_PAIRS", None)
    assert set(st.layer_kernels()) == {"conv3x3_mfma"}        # the path under test: a launch per arriving row (pair)
    x = input_tensor(wl, "cuda:0")
    H = wl["in_h"]
    outs = [[] for _ in range(wl["streams"])]
    for sample in range(2):                       # two samples back to back: the end of one, the start of the next
        r = 0
        while r < H:
            n = min(seg, H - r)
            st.push_segment(x[:, r:r + n].contiguous())
            r += n
            if reads_between and (r // seg) % 3 == 0:
                out, first, cnt = st.read_outputs(int(st.sizes.out_h))
                o = out.cpu().numpy()
                for b in range(wl["streams"]):
                    outs[b].append(o[b, :cnt[b]].copy())
        out, first, cnt = st.read_outputs(int(st.sizes.out_h))
        o = out.cpu().numpy()
        for b in range(wl["streams"]):
            outs[b].append(o[b, :cnt[b]].copy())
    torch.cuda.synchronize()
    stats = [st.get_stats(b) for b in range(wl["streams"])]
    st.close(); net.destroy()
    return [np.concatenate(o) for o in outs], stats


CASES = [
    (3, dict(streams=5, size=20, channels=(16, 16, 32, 32))),
    (4, dict(streams=3, size=24, channels=(16, 16, 16, 16, 32, 32, 32, 32))),
    (5, dict(streams=3, size=40, channels=(16, 16, 32, 32, 32, 32, 32))),
    (3, dict(streams=2, size=17, channels=(16, 16, 32, 32))),          # odd sizes: a row and a column dropped by the pool
]


@pytest.mark.parametrize("cfg,kw", CASES)
@pytest.mark.parametrize("seg", [2, 3, 5])
def test_two_rows_per_launch_equals_one(cfg, kw, seg):
    wl = wl_mod.make(cfg, **kw)
    one, st_one = _run(wl, 1, pairs=True)               # pushes of one row never pair
    two, st_two = _run(wl, seg, pairs=True, reads_between=(seg == 3))
    off, _ = _run(wl, seg, pairs=False)
    for b in range(wl["streams"]):
        assert one[b].shape == two[b].shape == off[b].shape
        assert np.array_equal(one[b], two[b]), (b, np.abs(one[b].astype(np.float64) - two[b]).max())
        assert np.array_equal(one[b], off[b])
        for key in ("events_in", "macs"):
            assert np.array_equal(st_one[b][key], st_two[b][key]), (b, key)
    H_o = one[0].shape[0] // 2
    for b in range(wl["streams"]):                       # and the values are the conventional network's
        check_stream(wl, two[b][:H_o], b)
        check_stream(wl, two[b][H_o:], b)


@pytest.mark.parametrize("cfg,kw", CASES[:3])
def test_pairs_mixed_with_subsets_and_issued_counters(cfg, kw):
    """Paired launches next to what interrupts them -- pushes of some streams only (a launch per layer) --
    and the counters of issued multiply-adds, which the kernel that takes two rows must add up like the
    one that takes one."""
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(cfg, **kw)
    B, H = wl["streams"], wl["in_h"]
    x = input_tensor(wl, "cuda:0")
    net = idf.net_from_workload(wl)

    def run(seg, mixed):
        st = idf.Streams(net, B, max_seg_rows=max(seg, 2))
        st.count_issued_macs(True)
        r, k = 0, 0
        while r < H:
            n = min(seg, H - r)
            if mixed and k % 3 == 1 and B > 1:      # the same rows as two pushes of some streams each
                ids_a, ids_b = list(range(0, B, 2)), list(range(1, B, 2))
                st.push_segment(x[ids_a, r:r + n].contiguous(), stream_ids=ids_a)
                st.push_segment(x[ids_b, r:r + n].contiguous(), stream_ids=ids_b)
            else:
                st.push_segment(x[:, r:r + n].contiguous())
            r += n; k += 1
        out, first, cnt = st.read_outputs(int(st.sizes.out_h))
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        res = [o[b, :cnt[b]].copy() for b in range(B)]
        iss = [st.get_issued_macs(b) for b in range(B)]
        stats = [st.get_stats(b) for b in range(B)]
        st.close()
        return res, iss, stats

    one, iss_one, st_one = run(1, False)
    two, iss_two, st_two = run(2, False)
    for b in range(B):
        assert np.array_equal(one[b], two[b])
        assert np.array_equal(iss_one[b], iss_two[b])
        assert np.array_equal(st_one[b]["macs"], st_two[b]["macs"])
    mix, _, _ = run(2, True)
    for b in range(B):
        assert np.array_equal(one[b], mix[b]), b
    net.destroy()
