"""Pins for the streaming (event-by-event) half of the CPU oracle and for the
paper-literal eager scheme: the paper's invariants, its Fig. 1 figure, counting
identities and brute force.  CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads as wl_mod
from oracle.eager import EagerNet
from workloads import conv, maxpool

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_stream(w, b, seg_rows=None, emit_round=None):
    integer = w["precision"] == "i8"
    return oracle.stream_run(w["layers"], w["x"][b], w["weights"], w["biases"],
                             seg_rows=seg_rows or w["seg_rows"], integer=integer, emit_round=emit_round)


def run_dense(w, b, emit_round=None, return_layers=False):
    integer = w["precision"] == "i8"
    return oracle.dense(w["layers"], w["x"][b], w["weights"], w["biases"], integer=integer,
                        emit_round=emit_round, return_layers=return_layers)


SMALL = {
    1: dict(streams=2, length=300),
    2: dict(streams=2, length=700, channels=(8, 8, 16, 16, 16, 16)),
    3: dict(streams=2, size=16, channels=(8, 8, 16, 16)),
    4: dict(streams=2, size=40, channels=(4, 4, 8, 8, 16, 16, 16, 16)),
    5: dict(streams=1, size=24, channels=(8, 8, 16, 16, 32, 32, 32)),
}


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_streaming_equals_layer_by_layer(cfg):
    """The paper's central claim: the incremental output is identical to the conventional one."""
    w = wl_mod.make(cfg, **SMALL[cfg])
    for b in range(w["streams"]):
        d = run_dense(w, b)
        e, st = run_stream(w, b)
        assert e.shape == d.shape == wl_mod.output_shape(w)
        if w["precision"] == "i8":
            assert np.array_equal(e, d)
        else:
            assert np.max(np.abs(e - d)) <= 1e-12 * max(1.0, np.max(np.abs(d)))
        assert np.abs(d).max() > 0
        # never more than K_h rows of a conv layer (1 of a pool) alive at once
        for L, p in zip(w["layers"], st["peak_rows"]):
            assert p <= (L["k_h"] if L["kind"] == "conv" else 1)


@pytest.mark.parametrize("seg", [1, 3, 16, 1000])
def test_segment_length_does_not_matter(seg):
    w = wl_mod.make(2, **SMALL[2])
    d = run_dense(w, 0)
    e, _ = run_stream(w, 0, seg_rows=seg)
    assert np.max(np.abs(e - d)) <= 1e-12 * np.max(np.abs(d))


def test_streaming_with_bf16_emission_equals_dense_with_bf16_emission():
    w = wl_mod.make(5, **SMALL[5])
    d = run_dense(w, 0, emit_round="bf16")
    e, _ = run_stream(w, 0, emit_round="bf16")
    # every emitted value is the same bf16 number on both sides unless a sum sits
    # within rounding of a bf16 tie; at this size none does
    assert np.max(np.abs(e - d)) <= 1e-9 * np.max(np.abs(d))
    assert np.max(np.abs(d - run_dense(w, 0))) > 0      # the rounding is really applied


def test_fig1_peak_stored_activations():
    """Fig. 1: K=3, K=3, one averaging output neuron: 7 activations at most, whatever the length."""
    golden = int([l for l in open(os.path.join(GOLDEN, "fig1_peak_activations.txt"))
                  if not l.startswith("#")][0])
    layers = [conv(1, 1, 3, 1), conv(1, 1, 3, 1)]
    ws = [np.ones((1, 1, 3, 1)), np.ones((1, 1, 3, 1))]
    # a sample must be at least 7 long for the second layer to have 3 outputs at all
    for length in (7, 8, 64, 4096):
        x = np.random.default_rng(length).random((length, 1, 1)) + 0.5
        s = oracle.Stream(layers, length, 1, 1, ws, avg_head=True)
        for r in range(length):
            s.push(x[r:r + 1])
        st = s.stats()
        assert st["peak_cells"] == golden == 3 + 3 + 1
        assert st["peak_rows"].tolist() == [3, 3]
        rows, mean = s.head()
        d = oracle.dense(layers, x, ws)
        assert rows == d.shape[0]
        assert abs(mean[0] - d.mean()) <= 1e-12 * abs(d.mean())


def test_1d_state_independent_of_length():
    w0 = wl_mod.make(2, streams=1, length=400, channels=(4, 4, 4, 4, 4, 4))
    peaks = []
    for length in (200, 4000, 100000):
        w = wl_mod.make(2, streams=1, length=length, channels=(4, 4, 4, 4, 4, 4))
        s = oracle.Stream(w["layers"], 0, 1, 1, w0["weights"])       # unbounded stream
        for r in range(0, length, 1000):
            s.push(w["x"][0, r:r + 1000])
            s.take()
        st = s.stats()
        peaks.append((st["peak_rows"].tolist(), st["peak_cells"]))
    # rows in flight per layer: ceil(K/s); the total never exceeds their sum (x 4 channels)
    assert peaks[0][0] == peaks[1][0] == peaks[2][0] == [9, 5, 9, 5, 9, 9]
    assert peaks[1][1] == peaks[2][1] == 4 * (9 + 5 + 9 + 5 + 9 + 9)
    assert peaks[0][1] <= peaks[1][1]


def test_2d_state_independent_of_height_and_linear_in_width():
    rng = np.random.default_rng(3)
    layers = [conv(1, 2, 3, 3, p_h=1, p_w=1), conv(2, 2, 3, 3, p_h=1, p_w=1), maxpool(2),
              conv(2, 3, 3, 3, p_h=1, p_w=1)]
    ws = [None if L["kind"] != "conv" else rng.normal(size=(L["c_out"], L["c_in"], 3, 3)) for L in layers]

    def peak(h, wd):
        x = rng.random((h, wd, 1)) + 0.1
        _, st = oracle.stream_run(layers, x, ws)
        return st["peak_cells"]
    assert peak(8, 8) == peak(32, 8) == peak(128, 8)
    assert peak(16, 16) == 2 * peak(16, 8) and peak(16, 32) == 4 * peak(16, 8)
    # the bound: K_h rows per conv layer plus one held row per pool
    assert peak(16, 8) <= 3 * 8 * 2 + 3 * 8 * 2 + 8 * 2 + 3 * 4 * 3


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_zero_input_costs_nothing(cfg):
    w = wl_mod.make(cfg, **SMALL[cfg])
    w["x"][:] = 0
    e, st = run_stream(w, 0)
    assert st["events_in"].sum() == 0 and st["macs"].sum() == 0
    assert not e.any()


def test_counts_events_and_macs():
    """Events into layer n = non-zeros of layer n-1's activations; executed multiply-adds =
    sum over those of (taps landing inside the output) x C_out."""
    w = wl_mod.make(3, streams=1, size=12, channels=(4, 4, 6, 6))
    d, per_layer = run_dense(w, 0, return_layers=True)
    _, st = run_stream(w, 0)
    acts = [w["x"][0]] + per_layer
    shapes = oracle.layer_shapes(w["layers"], w["in_h"], w["in_w"])
    for n, L in enumerate(w["layers"]):
        a = acts[n]
        assert st["events_in"][n] == np.count_nonzero(a)
        if L["kind"] != "conv":
            assert st["macs"][n] == 0
            continue
        H_o, W_o, _ = shapes[n]
        macs = 0
        for y, x, _ci in np.argwhere(a != 0):
            ty = sum(1 for ky in range(L["k_h"]) if (y + L["p_h"] - ky) % L["s_h"] == 0
                     and 0 <= (y + L["p_h"] - ky) // L["s_h"] < H_o)
            tx = sum(1 for kx in range(L["k_w"]) if (x + L["p_w"] - kx) % L["s_w"] == 0
                     and 0 <= (x + L["p_w"] - kx) // L["s_w"] < W_o)
            macs += ty * tx * L["c_out"]
        assert st["macs"][n] == macs


def test_single_impulse_touches_only_its_cone():
    layers = [conv(1, 2, 3, 3, p_h=1, p_w=1, act="none"), conv(2, 1, 3, 3, p_h=1, p_w=1, act="none")]
    ws = [np.ones((2, 1, 3, 3)), np.ones((1, 2, 3, 3))]
    x = np.zeros((15, 15, 1)); x[7, 6, 0] = 2.0
    e, st = oracle.stream_run(layers, x, ws)
    assert st["events_in"].tolist() == [1, 9 * 2]
    assert st["macs"].tolist() == [9 * 2, 18 * 9]
    nz = np.argwhere(e[:, :, 0] != 0)
    assert (nz.min(0) == [5, 4]).all() and (nz.max(0) == [9, 8]).all() and len(nz) == 25


def test_brute_force_all_small_inputs():
    """Every input over {0,1,2} of length 6 through a tiny integer net: dense, streaming and
    eager agree exactly."""
    rng = np.random.default_rng(0)
    layers = [conv(1, 2, 3, 1, p_h=1), conv(2, 2, 2, 1, s=2), conv(2, 1, 2, 1, act="none")]
    ws = [rng.integers(-3, 4, size=(L["c_out"], L["c_in"], L["k_h"], 1)) for L in layers]
    bs = [rng.integers(-2, 3, size=(L["c_out"],)) for L in layers]
    for vals in itertools.product((0, 1, 2), repeat=6):
        x = np.array(vals, dtype=np.int64).reshape(6, 1, 1)
        d = oracle.dense(layers, x, ws, bs, integer=True)
        e, _ = oracle.stream_run(layers, x, ws, bs, integer=True, seg_rows=1 + sum(vals) % 3)
        g = EagerNet(layers, 6, 1, 1, ws, bs, dtype=np.int64)
        for y in range(6):
            g.present_row(y, x[y])
        assert np.array_equal(d, e) and np.array_equal(d, g.announced[-1])


@pytest.mark.parametrize("with_bias", [False, True])
def test_eager_scheme_tracks_dense_after_every_row(with_bias):
    """After any prefix of the rows the eager net's announced activations equal the conventional
    net on the input seen so far, rest zero (the accumulated output of Fig. 3)."""
    rng = np.random.default_rng(4)
    layers = [conv(2, 3, 3, 3, p_h=1, p_w=1), conv(3, 3, 3, 3, p_h=1, p_w=1), maxpool(3),
              conv(3, 2, 3, 3, p_h=1, p_w=1)]
    ws = [None if L["kind"] != "conv" else rng.normal(size=(L["c_out"], L["c_in"], 3, 3)) for L in layers]
    bs = [None if (L["kind"] != "conv" or not with_bias) else rng.normal(size=(L["c_out"],)) * 0.3
          for L in layers]
    x = rng.random((8, 8, 2)); x[rng.random((8, 8)) < 0.5] = 0
    g = EagerNet(layers, 8, 8, 2, ws, bs)
    for y in range(8):
        g.present_row(y, x[y])
        partial = x.copy(); partial[y + 1:] = 0
        _, per_layer = oracle.dense(layers, partial, ws, bs, return_layers=True)
        for a, ref in zip(g.announced[1:], per_layer):
            assert np.max(np.abs(a - ref)) <= 1e-12
    final, _ = oracle.stream_run(layers, x, ws, bs)
    assert np.max(np.abs(g.announced[-1] - final)) <= 1e-12
    if not with_bias:
        # eager emission re-sends: it can only emit at least as many events as row-complete emission
        _, st = oracle.stream_run(layers, x, ws, bs)
        assert g.events[0] == st["events_in"][0]
        assert all(g.events[n] >= st["events_in"][n] for n in range(1, len(layers)))


def test_eager_1d_strided_int():
    rng = np.random.default_rng(6)
    layers = [conv(1, 2, 3, 1), conv(2, 2, 3, 1, s=2), maxpool(2, k_w=1), conv(2, 1, 2, 1, act="none")]
    ws = [None if L["kind"] != "conv" else rng.integers(-3, 4, size=(L["c_out"], L["c_in"], L["k_h"], 1))
          for L in layers]
    x = rng.integers(0, 4, size=(30, 1, 1))
    g = EagerNet(layers, 30, 1, 1, ws, dtype=np.int64)
    for y in range(30):
        g.present_row(y, x[y])
        partial = x.copy(); partial[y + 1:] = 0
        assert np.array_equal(g.announced[-1], oracle.dense(layers, partial, ws, integer=True))
    e, _ = oracle.stream_run(layers, x, ws, integer=True, seg_rows=4)
    assert np.array_equal(e, g.announced[-1])


def test_two_samples_back_to_back_rearm():
    w = wl_mod.make(3, streams=2, size=10, channels=(4, 4, 4, 4))
    s = oracle.Stream(w["layers"], 10, 10, 3, w["weights"])
    for b in range(2):
        for r in range(10):
            s.push(w["x"][b, r:r + 1])
        out = s.take()
        assert np.max(np.abs(out - run_dense(w, b))) <= 1e-12


def test_bad_descriptions_are_rejected():
    with pytest.raises(ValueError):
        oracle.dense([conv(2, 3, 3, 1)], np.zeros((8, 1, 1)), [np.zeros((3, 2, 3, 1))])   # channel mismatch
    with pytest.raises(ValueError):
        oracle.Stream([conv(1, 1, 3, 1, p_h=1)], 0, 1, 1, [np.zeros((1, 1, 3, 1))])       # unbounded + padding
