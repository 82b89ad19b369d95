"""Column-wise presentation (Fig. 2: row by row or column by column): the same network fed one
image column at a time gives the conventional network's output, column by column."""
import numpy as np
import pytest

import oracle
import workloads as wl_mod
from workloads import conv, maxpool
from helpers import TOL, rel_err

pytestmark = pytest.mark.gpu


def _net(prec, rng, H, W):
    q = dict(act="relu_shr_clamp", shr=3, clamp_hi=15) if prec == "i8" else {}
    # kernels that are not square, a stride along one axis only and padding that differs per axis:
    # any confusion of the two axes changes the result
    layers = [conv(2, 16, 3, 3, p_h=1, p_w=1, **q), conv(16, 16, 3, 3, p_h=1, p_w=1, **q), maxpool(16),
              conv(16, 16, 1, 3, p_h=0, p_w=1, **q), conv(16, 8, 3, 2, s=1, p_h=1, p_w=0, **({"act": "relu"} if prec == "i8" else {}))]
    layers[3]["s_w"] = 2
    ws, bs = [], []
    for L in layers:
        if L["kind"] != "conv":
            ws.append(None); bs.append(None); continue
        shape = (L["c_out"], L["c_in"], L["k_h"], L["k_w"])
        if prec == "i8":
            ws.append(rng.integers(-4, 5, size=shape).astype(np.int8)); bs.append(None)
        else:
            ws.append(rng.normal(0, 0.3, size=shape).astype(np.float32))
            bs.append(rng.normal(0, 0.2, size=(L["c_out"],)).astype(np.float32))
    x = rng.integers(0, 8, size=(3, H, W, 2)).astype(np.int8) if prec == "i8" else rng.random((3, H, W, 2)).astype(np.float32)
    x[rng.random((3, H, W)) < 0.5] = 0
    return dict(name="colwise", precision=prec, in_h=H, in_w=W, in_c=2, layers=layers, weights=ws, biases=bs, x=x,
                seg_rows=1, streams=3)


@pytest.mark.parametrize("prec,seg", [("f32", 1), ("i8", 1), ("f32", 3)])
def test_columns_in_columns_out(prec, seg):
    import torch
    import paper_1804_10727_amd as idf
    H, W = 12, 22
    wl = _net(prec, np.random.default_rng(21), H, W)
    net = idf.net_from_workload(wl, columnwise=True)
    st = idf.Streams(net, 3, max_seg_rows=seg)
    want = [oracle.dense(wl["layers"], wl["x"][b], wl["weights"], wl["biases"], integer=prec == "i8") for b in range(3)]
    oh, ow, oc = want[0].shape
    assert (st.sizes.out_h, st.sizes.out_w, st.sizes.out_c) == (ow, oh, oc)      # columns per sample, rows of the map
    xt = torch.from_numpy(np.ascontiguousarray(wl["x"].transpose(0, 2, 1, 3))).to("cuda:0")    # [stream][column][row][c]
    cols = [[] for _ in range(3)]
    for c0 in range(0, W, seg):
        n = min(seg, W - c0)
        st.push_segment(xt[:, c0:c0 + n].contiguous())
        out, first, cnt = st.read_outputs(8)
        o = out.cpu().numpy()
        for b in range(3):
            cols[b].append(o[b, :cnt[b]])
    for b in range(3):
        g = np.concatenate(cols[b]).transpose(1, 0, 2)           # back to [row][column][c]
        assert g.shape == want[b].shape
        if prec == "i8":
            assert np.array_equal(g.astype(np.int64), want[b]), b
        else:
            assert rel_err(g, want[b]) <= TOL["f32"], b
    st.close(); net.destroy()


def test_column_length_is_what_the_state_scales_with():
    import paper_1804_10727_amd as idf
    wl = _net("f32", np.random.default_rng(2), 12, 22)
    a = idf.net_from_workload(wl, columnwise=True).query_sizes(1)
    wl2 = _net("f32", np.random.default_rng(2), 12, 44)           # twice as many columns: same state
    b = idf.net_from_workload(wl2, columnwise=True).query_sizes(1)
    wl3 = _net("f32", np.random.default_rng(2), 24, 22)           # columns twice as long: about twice the state
    c = idf.net_from_workload(wl3, columnwise=True).query_sizes(1)
    assert a.state_bytes_per_stream == b.state_bytes_per_stream
    assert 1.8 * a.state_bytes_per_stream <= c.state_bytes_per_stream <= 2.2 * a.state_bytes_per_stream
