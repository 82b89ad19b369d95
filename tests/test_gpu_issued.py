"""GPU checks of the issued multiply-add counter: what the compaction of events (Sec. 1: zero
values cause no arithmetic) leaves for the kernels to do.  Executed multiply-adds are checked
against the oracle elsewhere; here the issued count is held to what it must be by construction."""
import numpy as np
import pytest

import workloads as wl_mod
from helpers import check_stream, gpu_run

pytestmark = pytest.mark.gpu


def _counts(wl, seg_rows=None, events_per_step=None, want_out=False):
    """events_per_step: idf_set_event_path's argument -- 0 or None (the library's setting after
    open): the contraction on the matrix cores always; large: the event list on the vector units
    whenever the tile's events fit the list."""
    out, st, net = gpu_run(wl, seg_rows, return_streams=True, count_issued=True, events_per_kstep=events_per_step)
    B = wl["streams"]
    issued = [st.get_issued_macs(b) for b in range(B)]
    stats = [st.get_stats(b) for b in range(B)]
    kinds = st.layer_kernels()
    st.close(); net.destroy()
    if want_out:
        return issued, stats, kinds, out
    return issued, stats, kinds


def _mfma_steps(c_in, vl):
    return (3 * c_in + 2 * vl - 1) // (2 * vl)


def test_matrix_core_path_issues_between_executed_and_dense_tiles():
    wl = wl_mod.make(4, streams=3, size=40, channels=(16, 16, 16, 16, 32, 32, 32, 32))
    issued, stats, kinds = _counts(wl, events_per_step=0)
    assert all(k in ("conv3x3_mfma", "pool_fused") or "mfma" in k or "pool" in k for k in kinds)
    w = 40
    for b in range(3):
        width = w
        for l, L in enumerate(wl["layers"]):
            if L["kind"] != "conv":
                assert issued[b][l] == 0
                width //= 2
                continue
            # every K-step of every 32 x 32 tile of every arriving row, three kernel rows each
            steps = _mfma_steps(L["c_in"], 16)
            tiles = -(-width // 32) * -(-L["c_out"] // 32)
            bound = width * tiles * steps * 3 * 32 * 32 * 32      # rows of the layer's input = its width (square maps)
            assert stats[b]["macs"][l] <= issued[b][l] <= bound, (b, l)
    # 80 % of the input is zero: the first layers skip most steps
    assert sum(int(i[1]) for i in issued) < 0.6 * 3 * 40 * 2 * _mfma_steps(16, 16) * 3 * 32 * 32 * 32


def test_dense_input_issues_every_step_and_zero_input_none():
    wl = wl_mod.make(4, streams=2, size=32, channels=(16, 16, 16, 16, 16, 16, 16, 16))
    dense = dict(wl); dense["x"] = np.full_like(wl["x"], 3)
    issued, stats, _ = _counts(dense, events_per_step=0)
    # layer 0: one input channel, 32 rows of 32 positions, one tile, one K-step, three kernel rows
    for b in range(2):
        assert issued[b][0] == 32 * 1 * 1 * 3 * 32 * 32 * 32
    # nothing but zeros: no layer executes anything; the first layer (one input channel: its one
    # K-step is always visited) still issues its step, every layer behind it skips everything
    zero = dict(wl); zero["x"] = np.zeros_like(wl["x"])
    issued, stats, _ = _counts(zero, events_per_step=0)
    for b in range(2):
        assert int(stats[b]["macs"].sum()) == 0
        assert issued[b][0] == 32 * 1 * 1 * 3 * 32 * 32 * 32 and int(issued[b][1:].sum()) == 0
    # with the event path switched on (a first layer of one channel then always takes it) zeros cost
    # nothing anywhere
    issued, stats, _ = _counts(zero, events_per_step=8)
    for b in range(2):
        assert int(stats[b]["macs"].sum()) == 0 and int(issued[b].sum()) == 0


@pytest.mark.parametrize("size,channels", [(40, (16, 16, 16, 16, 32, 32, 32, 32)), (70, (16, 16, 32, 32, 64, 64, 64, 64))])
def test_event_list_path_and_contraction_agree_bit_for_bit(size, channels):
    """int8 tiles go one of two ways: packed event list on the vector units (ballot-free prefix sum per
    position, one weight word and three multiply-adds per event and output channel) or contraction on
    the matrix cores.  Forced either way, and mixed by a limit of 8 events per K-step, outputs and counters are the same
    integers, equal to the oracle's; the event path issues exactly the events' taps times the tile's
    channel width: never more than three times what the contraction issues at this density, far less
    where the input is sparse."""
    wl = wl_mod.make(4, streams=3, size=size, channels=channels)
    i_m, s_m, _, o_m = _counts(wl, events_per_step=0, want_out=True)
    i_e, s_e, _, o_e = _counts(wl, events_per_step=100000, want_out=True)
    i_d, s_d, _, o_d = _counts(wl, events_per_step=8, want_out=True)
    assert np.array_equal(o_m, o_e) and np.array_equal(o_m, o_d)
    for b in range(3):
        check_stream(wl, o_e[b], b)
        assert s_m[b]["events_in"].tolist() == s_e[b]["events_in"].tolist() == s_d[b]["events_in"].tolist()
        assert s_m[b]["macs"].tolist() == s_e[b]["macs"].tolist() == s_d[b]["macs"].tolist()
        for l, L in enumerate(wl["layers"]):
            if L["kind"] != "conv":
                continue
            assert s_e[b]["macs"][l] <= i_e[b][l] and s_d[b]["macs"][l] <= i_d[b][l]
            # an event visited by three output positions, three kernel rows, a tile 32 channels wide:
            # 9 * 32 per event and channel chunk at most, and nothing for the zeros (layers of up to 16
            # input channels; wider ones always take the contraction)
            chunks = -(-L["c_out"] // 32)
            if L["c_in"] <= 16:
                assert i_e[b][l] <= s_e[b]["events_in"][l] * 9 * 32 * chunks
            else:
                assert i_e[b][l] == i_m[b][l]
        # the first layer (one input channel): the contraction pads its K from 3 to 32 and its 16 channels to 32
        assert i_d[b][0] == i_e[b][0] and i_e[b][0] * 8 < i_m[b][0]
        assert int(i_d[b].sum()) <= int(i_m[b].sum())


def test_cascade_issues_all_rows_of_channels_with_events():
    wl = wl_mod.make(2, streams=3, length=320, channels=(8, 8, 16, 16, 32, 64))
    issued, stats, kinds = _counts(wl)
    assert all(k == "cascade1d" for k in kinds)
    for b in range(3):
        for l in range(6):
            assert stats[b]["macs"][l] <= issued[b][l]
    # an input without zeros: every push of 16 rows visits the one input channel of layer 0 and
    # computes 16 rows x 9 taps for each of its 8 output channels
    dense = dict(wl); dense["x"] = np.abs(wl["x"]) + 1.0
    issued, stats, _ = _counts(dense)
    for b in range(3):
        assert issued[b][0] == (320 // 16) * 16 * 9 * 8
    zero = dict(wl); zero["x"] = np.zeros_like(wl["x"])
    issued, _, _ = _counts(zero)
    assert all(int(i.sum()) == 0 for i in issued)
