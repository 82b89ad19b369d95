"""idf_open_streams_static: streams whose workspace is the library's own static device array (for
callers that cannot allocate device memory) give what idf_open_streams gives -- the same kernels on
other memory, so bit for bit -- call after call, also when the next streams are smaller and find the
previous ones' bytes in the array."""
import numpy as np
import pytest

import workloads as wl_mod

pytestmark = pytest.mark.gpu


def run(wl, seg, static):
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, wl["streams"], max_seg_rows=seg, static_workspace=static)
    assert (st.workspace is None) == static
    x = input_tensor(wl)
    for r in range(0, wl["in_h"], seg):
        st.push_segment(x[:, r:r + seg].contiguous())
    out, first, cnt = st.read_outputs(int(st.sizes.out_h))
    torch.cuda.synchronize()
    stats = [st.get_stats(b) for b in range(wl["streams"])]
    st.close()
    net.destroy()
    assert (first == 0).all() and (cnt == st.sizes.out_h).all()
    return out.cpu().numpy(), stats


def test_static_workspace_matches_caller_workspace_twice_second_smaller():
    from helpers import check_stream
    cases = [
        (wl_mod.make(4, streams=6, size=48, channels=(16, 16, 16, 16, 32, 32, 32, 32)), 1),   # int8, matrix-core kernel, staged rows
        (wl_mod.make(3, streams=3, size=16, channels=(16, 16, 32, 32)), 1),                  # smaller: float32
        (wl_mod.make(2, streams=2, length=320, channels=(8, 8, 16, 16, 16, 16)), 16),        # 1-D cascade, smaller still
    ]
    for wl, seg in cases:
        print(f"static workspace: {wl['name']} streams={wl['streams']}", flush=True)
        want, want_stats = run(wl, seg, static=False)
        got, got_stats = run(wl, seg, static=True)
        assert got.dtype == want.dtype and got.shape == want.shape
        assert np.array_equal(got, want)                    # same kernels, same order: identical bits
        for a, b in zip(got_stats, want_stats):
            assert np.array_equal(a["events_in"], b["events_in"]) and np.array_equal(a["macs"], b["macs"])
        check_stream(wl, got[0], 0)                          # and both are right: against the oracle
        check_stream(wl, got[-1], wl["streams"] - 1)


def test_static_workspace_refusals():
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd import binding
    wl = wl_mod.make(3, streams=2, size=16, channels=(16, 16, 32, 32))
    net = idf.net_from_workload(wl)
    a = idf.Streams(net, 2, static_workspace=True)
    with pytest.raises(idf.IdfError) as e:                  # the array is taken
        idf.Streams(net, 2, static_workspace=True)
    assert e.value.code == binding.IDF_ESTATE
    a.close()
    b = idf.Streams(net, 2, static_workspace=True)          # free again after close
    b.close()
    net.destroy()
    big = wl_mod.make(5, streams=1)                         # 64 streams of the largest configuration: far beyond the array
    netb = idf.net_from_workload(big)
    assert netb.query_sizes(64, 1, 0).workspace_bytes > (32 << 20)
    with pytest.raises(idf.IdfError) as e:
        idf.Streams(netb, 64, static_workspace=True)
    assert e.value.code == binding.IDF_ENOMEM and "static" in str(e.value)
    netb.destroy()
