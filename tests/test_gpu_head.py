"""GPU parity for the averaging output units (Fig. 1; Sec. 4: output units whose value settles as
rows come in): running per-channel mean of the last layer's completed rows, against the oracle's
head fed the same rows, at several points of the presentation."""
import numpy as np
import pytest

import oracle
import workloads as wl_mod
from helpers import TOL

pytestmark = pytest.mark.gpu


def _oracle_stream(wl, b):
    return oracle.Stream(wl["layers"], wl["in_h"], wl["in_w"], wl["in_c"], wl["weights"], wl["biases"],
                         integer=wl["precision"] == "i8",
                         emit_round="bf16" if wl["precision"] == "bf16" else None, avg_head=True)


def _check(wl, seg, read_at, exact):
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    B, H = wl["streams"], wl["in_h"]
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, B, max_seg_rows=seg)
    st.enable_head()
    ref = [_oracle_stream(wl, b) for b in range(B)]
    x = input_tensor(wl)
    seen_nonzero = False
    for i, r in enumerate(range(0, H, seg)):
        st.push_segment(x[:, r:r + seg].contiguous())
        for b in range(B):
            ref[b].push(wl["x"][b, r:r + seg])
        if i in read_at or r + seg >= H:
            rows, mean = st.read_head()
            for b in range(B):
                o_rows, o_mean = ref[b].head()
                assert rows[b] == o_rows
                scale = max(float(np.max(np.abs(o_mean))), 1e-30)
                err = float(np.max(np.abs(mean[b] - o_mean))) / scale
                assert err <= (1e-12 if exact else (2e-2 if wl["precision"] == "bf16" else TOL["f32"])), (i, b, err)
                seen_nonzero |= o_rows > 0 and scale > 1e-20
        if i == 1:      # reading outputs in between must not disturb the units
            st.read_outputs(4)
    assert seen_nonzero
    st.close(); net.destroy()


def test_fig1_net_one_sample_per_push():
    # the two-layer K=3 net of Fig. 1 with its averaging output neuron, one sample at a time
    from workloads import conv
    rng = np.random.default_rng(5)
    layers = [conv(1, 1, 3, 1), conv(1, 1, 3, 1)]
    ws = [(np.abs(rng.normal(size=(1, 1, 3, 1))) + 0.1).astype(np.float32) for _ in layers]
    x = (rng.random((1, 60, 1, 1)) + 0.25).astype(np.float32)
    wl = dict(name="fig1", precision="f32", in_h=60, in_w=1, in_c=1, layers=layers, weights=ws,
              biases=[None, None], x=x, seg_rows=1, streams=1)
    _check(wl, 1, read_at={0, 3, 4, 5, 6, 20}, exact=False)


def test_1d_streams_in_segments():
    wl = wl_mod.make(2, streams=3, length=480, channels=(8, 8, 16, 16, 32, 32))
    _check(wl, 16, read_at={0, 2, 3, 9, 17}, exact=False)


def test_2d_int_exact_and_float():
    wl = wl_mod.make(4, streams=2, size=24, channels=(4, 4, 8, 8, 16, 16, 16, 16))
    _check(wl, 1, read_at={5, 12, 20, 23}, exact=True)
    wl = wl_mod.make(3, streams=3, size=16, channels=(8, 8, 16, 16))
    _check(wl, 2, read_at={1, 3, 6}, exact=False)


def test_head_restarts_with_the_next_sample_and_needs_enabling():
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    wl = wl_mod.make(3, streams=4, size=12, channels=(8, 8, 8, 8))
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, 2)
    with pytest.raises(idf.IdfError):
        st.read_head()
    st.enable_head()
    x = input_tensor(wl)
    for sample in range(2):
        for r in range(12):
            st.push_segment(x[2 * sample:2 * sample + 2, r:r + 1].contiguous())
            if sample == 1 and r == 6:
                st.read_outputs(64)          # the first sample's rows leave the output area
        rows, mean = st.read_head()
        for i in range(2):
            ref = _oracle_stream(wl, 2 * sample + i)
            ref.push(wl["x"][2 * sample + i])
            o_rows, o_mean = ref.head()
            assert rows[i] == o_rows == st.sizes.out_h
            assert np.max(np.abs(mean[i] - o_mean)) <= TOL["f32"] * np.max(np.abs(o_mean))
    st.push_segment(x[0:2, 0:1].contiguous())
    with pytest.raises(idf.IdfError):
        st.enable_head()
    st.close(); net.destroy()


@pytest.mark.parametrize("cfg,kw,seg", [
    (3, dict(streams=3, size=16, channels=(16, 16, 32, 32)), 1),
    (4, dict(streams=2, size=48, channels=(16, 16, 16, 16, 16, 16, 16, 16)), 2),
])
def test_fully_connected_output_units_settle_row_by_row(cfg, kw, seg):
    """Ten class units over the last layer's map: after every few rows their values are the bias
    plus the weighted sum of the rows completed so far; after the last row, the conventional
    network's fully connected layer (Sec. 4, Fig. 3 / Fig. 4)."""
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    from helpers import oracle_dense
    wl = wl_mod.make(cfg, **kw)
    B, H = wl["streams"], wl["in_h"]
    rng = np.random.default_rng(9)
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, B, max_seg_rows=seg)
    oh, ow, oc = int(st.sizes.out_h), int(st.sizes.out_w), int(st.sizes.out_c)
    w = rng.normal(0, 1.0 / np.sqrt(oh * ow * oc), size=(10, oh, ow, oc)).astype(np.float32)
    b = rng.normal(0, 0.1, size=(10,)).astype(np.float32)
    st.enable_head_units(w, b)
    dense = [oracle_dense(wl, s).astype(np.float64) for s in range(B)]
    x = input_tensor(wl)
    rows0, v0 = st.read_head_units()
    assert (rows0 == 0).all() and np.allclose(v0, b[None, :].astype(np.float64))
    seen = set()
    for i, r in enumerate(range(0, H, seg)):
        st.push_segment(x[:, r:r + seg].contiguous())
        if True:
            rows, vals = st.read_head_units()
            for s in range(B):
                want = oracle.head_units(dense[s][:rows[s]], w, b)
                assert np.max(np.abs(vals[s] - want)) <= 1e-5 * max(1.0, np.max(np.abs(want))), (i, s)
                seen.add(int(rows[s]))
    assert oh in seen and len(seen) >= 3
    for s in range(B):      # after the last row: the conventional network's dense layer on the whole map
        full = np.tensordot(w.astype(np.float64), dense[s], axes=([1, 2, 3], [0, 1, 2])) + b
        assert np.argmax(vals[s]) == np.argmax(full)
    with pytest.raises(idf.IdfError):
        st.snapshot(0)
    st.close(); net.destroy()


def test_convergence_curve_matches_the_oracle_row_by_row():
    """The accumulated-output curve of Sec. 4 (Fig. 3 / Fig. 4) as the package's script measures it:
    every point against the oracle's class units on the rows the dense oracle says are complete."""
    from paper_1804_10727_amd import convergence
    from helpers import oracle_dense
    wl = wl_mod.make(3, streams=6, size=16, channels=(16, 16, 32, 32))
    seen, vals, w, b = convergence.curve(wl, n_units=5, seed=4)
    dense = [oracle_dense(wl, s).astype(np.float64) for s in range(6)]
    assert seen[-1] == dense[0].shape[0] and (np.diff(seen) >= 0).all() and seen[0] == 0
    for r in range(wl["in_h"]):
        for s in range(6):
            want = oracle.head_units(dense[s][:seen[r]], w, b)
            assert np.max(np.abs(vals[r, s] - want)) <= 1e-5 * max(1.0, np.max(np.abs(want))), (r, s)
    table = convergence.summarise(seen, vals)
    assert table[-1][2] == 1.0 and table[-1][3] == 0.0           # after the last row: the conventional network
    assert table[0][3] > table[len(table) // 2][3] > 0.0          # and on the way the values close in on it
