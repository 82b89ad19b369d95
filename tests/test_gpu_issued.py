"""GPU checks of the issued multiply-add counter: what the compaction of events (Sec. 1: zero
values cause no arithmetic) leaves for the kernels to do.  Executed multiply-adds are checked
against the oracle elsewhere; here the issued count is held to what it must be by construction."""
import numpy as np
import pytest

import workloads as wl_mod
from helpers import gpu_run

pytestmark = pytest.mark.gpu


def _counts(wl, seg_rows=None):
    _, st, net = gpu_run(wl, seg_rows, return_streams=True, count_issued=True)
    B = wl["streams"]
    issued = [st.get_issued_macs(b) for b in range(B)]
    stats = [st.get_stats(b) for b in range(B)]
    kinds = st.layer_kernels()
    st.close(); net.destroy()
    return issued, stats, kinds


def _mfma_steps(c_in, vl):
    return (3 * c_in + 2 * vl - 1) // (2 * vl)


def test_matrix_core_path_issues_between_executed_and_dense_tiles():
    wl = wl_mod.make(4, streams=3, size=40, channels=(16, 16, 16, 16, 32, 32, 32, 32))
    issued, stats, kinds = _counts(wl)
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
    issued, stats, _ = _counts(dense)
    # layer 0: one input channel, 32 rows of 32 positions, one tile, one K-step, three kernel rows
    for b in range(2):
        assert issued[b][0] == 32 * 1 * 1 * 3 * 32 * 32 * 32
    # nothing but zeros: no layer executes anything; the first layer (one input channel: its one
    # K-step is always visited) still issues its step, every layer behind it skips everything
    zero = dict(wl); zero["x"] = np.zeros_like(wl["x"])
    issued, stats, _ = _counts(zero)
    for b in range(2):
        assert int(stats[b]["macs"].sum()) == 0
        assert issued[b][0] == 32 * 1 * 1 * 3 * 32 * 32 * 32 and int(issued[b][1:].sum()) == 0


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
