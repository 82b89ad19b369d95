"""GPU checks at the edges: calls with nothing or too much in them (turned into errors by the host,
nothing reaches a kernel), the smallest maps the kernels take, and the widest layers on either side of
what the matrix-core kernel serves."""
import numpy as np
import pytest

import workloads as wl_mod
from workloads import conv, maxpool
from helpers import check_stream, gpu_run

pytestmark = pytest.mark.gpu


def _net(prec, H, W, C0, layers, seed, streams=2, density=0.5, w_scale=None):
    rng = np.random.default_rng(seed)
    ws, bs = [], []
    for L in layers:
        if L["kind"] != "conv":
            ws.append(None); bs.append(None)
            continue
        shape = (L["c_out"], L["c_in"], L["k_h"], L["k_w"])
        if prec == "i8":
            ws.append(rng.integers(-7, 8, size=shape).astype(np.int8))      # symmetric: sums of hundreds of terms must not all be negative
        else:
            w = rng.normal(0.0, np.sqrt(2.0 / (L["c_in"] * L["k_h"] * L["k_w"])), size=shape).astype(np.float32)
            ws.append(wl_mod.round_to_bf16(w) if prec == "bf16" else w)
        bs.append(None)
    if prec == "i8":
        x = (rng.integers(1, 16, size=(streams, H, W, C0)) * (rng.random((streams, H, W, C0)) < density)).astype(np.int8)
    else:
        x = (rng.random((streams, H, W, C0)) * (rng.random((streams, H, W, C0)) < density)).astype(np.float32)
        if prec == "bf16":
            x = wl_mod.round_to_bf16(x)
    return dict(name="edge", precision=prec, in_h=H, in_w=W, in_c=C0, layers=layers, weights=ws, biases=bs, x=x,
                seg_rows=1, streams=streams)


def test_calls_with_nothing_or_too_much_in_them_are_errors():
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor, IDF_EINVAL, IDF_ESTATE
    wl = wl_mod.make(3, streams=3, size=16, channels=(16, 16, 16, 16))        # 16 rows in, 8 rows out
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 3, max_seg_rows=2, out_cap_rows=4)
    x = input_tensor(wl)

    def refused(code, fn):
        with pytest.raises(idf.IdfError) as e:
            fn()
        assert e.value.code == code, (e.value.code, str(e.value))

    refused(IDF_EINVAL, lambda: st.push_segment(x[:, 0:1].contiguous(), stream_ids=[]))          # no stream
    refused(IDF_EINVAL, lambda: st.push_segment(x[:, 0:1].contiguous(), n_rows=0))               # no row
    refused(IDF_EINVAL, lambda: st.push_segment(x[:, 0:3].contiguous()))                         # more rows than max_seg_rows
    refused(IDF_EINVAL, lambda: st.push_segment(x[:2, 0:1].contiguous(), stream_ids=[0, 0]))     # a stream twice
    refused(IDF_EINVAL, lambda: st.push_segment(x[:1, 0:1].contiguous(), stream_ids=[3]))        # no such stream
    refused(IDF_EINVAL, lambda: st.read_outputs(0))
    assert all(st.rows_pushed(b) == 0 for b in range(3))                                         # none of it left a trace
    # the output ring of four rows fills up: the push that would complete a fifth row is refused, a read makes room
    r = 0
    while True:
        try:
            st.push_segment(x[:, r:r + 1].contiguous())
        except idf.IdfError as e:
            assert e.code == IDF_ESTATE and "output area full" in str(e)
            break
        r += 1
    assert 0 < r < 16
    out, first, cnt = st.read_outputs(4)
    assert (cnt == 4).all() and (first == 0).all()
    for rr in range(r, 16):
        if rr == 15:                                                                               # one row left in the sample
            refused(IDF_ESTATE, lambda: st.push_segment(x[:, 14:16].contiguous()))
        st.push_segment(x[:, rr:rr + 1].contiguous())
        st.read_outputs(4)
    assert all(st.rows_pushed(b) == 0 for b in range(3))                                         # the sample is complete: re-armed
    torch.cuda.synchronize()
    st.close(); net.destroy()


@pytest.mark.parametrize("prec", ["i8", "f32", "bf16"])
def test_smallest_maps(prec):
    """Two rows of two positions: every tile is mostly padding, every row is first, last or both; a pool
    leaves a single value per channel."""
    q = dict(act="relu_shr_clamp", shr=3, clamp_hi=15) if prec == "i8" else {}
    c0 = 16 if prec != "f32" else 4
    layers = [conv(c0, 16, 3, 3, p_h=1, p_w=1, **q), maxpool(16), conv(16, 16, 3, 3, p_h=1, p_w=1, **({"act": "relu"} if prec == "i8" else {}))]
    wl = _net(prec, 2, 2, c0, layers, seed=21, streams=3, density=0.8)
    out = gpu_run(wl)
    assert out.shape[1:] == (1, 1, 16)
    for b in range(3):
        check_stream(wl, out[b], b)
    # and a single column of three rows in one dimension less: the generic kernels
    layers1 = [conv(c0, 16, 3, 1, **({"act": "relu"} if prec == "i8" else {}))]
    wl1 = _net(prec, 3, 1, c0, layers1, seed=22, streams=2, density=0.9)
    out1 = gpu_run(wl1)
    assert out1.shape[1:] == (1, 1, 16)
    for b in range(2):
        check_stream(wl1, out1[b], b)


@pytest.mark.parametrize("prec,c_in,want", [("bf16", 336, "conv3x3_mfma"), ("bf16", 352, "conv_generic"),
                                            ("i8", 672, "conv3x3_mfma"), ("i8", 704, "conv_generic")])
def test_widest_layers_either_side_of_the_matrix_core_limit(prec, c_in, want):
    """The matrix-core kernel takes up to 64 K-steps (63 here: 3 * c_in / 16 for bfloat16, / 32 for int8);
    one more 16-byte cell per position and the layer goes to the generic kernel.  Same results either way."""
    import paper_1804_10727_amd as idf
    q = dict(act="relu") if prec == "i8" else {}
    layers = [conv(c_in, 32, 3, 3, p_h=1, p_w=1, **q)]
    wl = _net(prec, 5, 9, c_in, layers, seed=c_in, streams=2, density=0.3)
    out, st, net = gpu_run(wl, return_streams=True)
    assert st.layer_kernels()[0].startswith(want), st.layer_kernels()
    st.close(); net.destroy()
    for b in range(2):
        check_stream(wl, out[b], b)
