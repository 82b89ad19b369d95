"""Pins for the dense (layer-by-layer) half of the CPU oracle: hand-worked values,
a library convolution, textbook identities.  CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads as wl_mod
from workloads import conv, maxpool


def torch_dense(layers, x, weights, biases, integer=False):
    """Same network through torch's CPU routines in float64 (exact for the small integers used)."""
    t = torch.from_numpy(np.asarray(x, dtype=np.float64)).permute(2, 0, 1)[None]   # 1,C,H,W
    for L, w, b in zip(layers, weights, biases):
        if L["kind"] == "conv":
            tw = torch.from_numpy(np.asarray(w, dtype=np.float64))
            tb = None if b is None else torch.from_numpy(np.asarray(b, dtype=np.float64))
            t = F.conv2d(t, tw, tb, stride=(L["s_h"], L["s_w"]), padding=(L["p_h"], L["p_w"]))
            if L["act"] in ("relu", "relu_shr_clamp"):
                t = F.relu(t)
            if L["act"] == "relu_shr_clamp":
                t = torch.clamp(torch.floor(t / (1 << L["shr"])), max=L["clamp_hi"])
        else:
            t = F.max_pool2d(t, kernel_size=(2, L["k_w"]), stride=(2, L["s_w"]))
    return t[0].permute(1, 2, 0).numpy()


def test_hand_worked_1d():
    # y[o] = sum_k w[k] x[o+k]; x = 1 0 2 0 0 3, w = 1 2 3
    #   o=0: 1*1+2*0+3*2 = 7   o=1: 0+2*2+0 = 4   o=2: 1*2+0+0 = 2   o=3: 0+0+3*3 = 9
    # bias -3 then ReLU: 4 1 0 6
    layers = [conv(1, 1, 3, 1)]
    x = np.array([1, 0, 2, 0, 0, 3], dtype=np.float64).reshape(6, 1, 1)
    w = [np.array([1, 2, 3], dtype=np.float64).reshape(1, 1, 3, 1)]
    out = oracle.dense(layers, x, w, [np.array([-3.0])])
    assert out.reshape(-1).tolist() == [4.0, 1.0, 0.0, 6.0]
    out_i = oracle.dense(layers, x, w, [np.array([-3])], integer=True)
    assert out_i.reshape(-1).tolist() == [4, 1, 0, 6]


def test_hand_worked_2d_impulse_orientation():
    # a single 1 in the centre of a 3x3 image, 3x3 kernel, same padding: output
    # pixel (oy,ox) sees the impulse through tap (ky,kx) = (1-oy+1, 1-ox+1), so
    # the output is the kernel rotated by 180 degrees.
    layers = [conv(1, 1, 3, 3, p_h=1, p_w=1, act="none")]
    x = np.zeros((3, 3, 1)); x[1, 1, 0] = 1.0
    k = np.arange(1, 10, dtype=np.float64).reshape(1, 1, 3, 3)
    out = oracle.dense(layers, x, [k])[:, :, 0]
    assert np.array_equal(out, k[0, 0, ::-1, ::-1])


def test_hand_worked_channels_and_stride():
    # 2 input channels, 1 output channel, K=2 stride 2 along rows, W=1:
    # rows (a,b): (1,2) (3,4) (5,6) (7,8); w[ci][ky] = [[1,10],[100,1000]]
    # o=0: 1*1 + 10*3 + 100*2 + 1000*4 = 4231 ; o=1: 5 + 70 + 600 + 8000 = 8675
    layers = [conv(2, 1, 2, 1, s=2, act="none")]
    x = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float64).reshape(4, 1, 2)
    w = np.array([[1, 10], [100, 1000]], dtype=np.float64).reshape(1, 2, 2, 1)
    out = oracle.dense(layers, x, [w])
    assert out.reshape(-1).tolist() == [4231.0, 8675.0]


def test_hand_worked_pool_and_requant():
    # relu -> >>4 -> clamp 15, then 2x2 max
    layers = [conv(1, 1, 1, 1, act="relu_shr_clamp", shr=4, clamp_hi=15), maxpool(1)]
    x = np.array([[-5, 31], [32, 47], [48, 1000], [15, 16]], dtype=np.int64).reshape(4, 2, 1)
    w = [np.array([1], dtype=np.int64).reshape(1, 1, 1, 1), None]
    out, per_layer = oracle.dense(layers, x, w, integer=True, return_layers=True)
    assert per_layer[0][:, :, 0].tolist() == [[0, 1], [2, 2], [3, 15], [0, 1]]
    assert out.reshape(-1).tolist() == [2, 15]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_torch_conv2d_float(seed):
    rng = np.random.default_rng(seed)
    layers = [conv(3, 5, 3, 3, p_h=1, p_w=1), conv(5, 4, 3, 3, s=2, p_h=1, p_w=1), maxpool(4),
              conv(4, 6, 5, 3, p_h=2, p_w=0, act="none"), conv(6, 2, 1, 1)]
    x = rng.normal(size=(23, 26, 3))
    x[rng.random(x.shape) < 0.4] = 0
    ws = [None if L["kind"] != "conv" else rng.normal(size=(L["c_out"], L["c_in"], L["k_h"], L["k_w"]))
          for L in layers]
    bs = [None if L["kind"] != "conv" or i == 1 else rng.normal(size=(L["c_out"],)) for i, L in enumerate(layers)]
    ref = torch_dense(layers, x, ws, bs)
    out = oracle.dense(layers, x, ws, bs)
    assert out.shape == ref.shape
    assert np.max(np.abs(out - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_against_torch_conv1d_strided():
    rng = np.random.default_rng(5)
    layers = [conv(1, 4, 9, 1), conv(4, 4, 9, 1, s=2), conv(4, 3, 9, 1), maxpool(3, k_w=1)]
    x = rng.normal(size=(200, 1, 1))
    ws = [None if L["kind"] != "conv" else rng.normal(size=(L["c_out"], L["c_in"], L["k_h"], 1)) for L in layers]
    ref = torch_dense(layers, x, ws, [None] * 4)
    out = oracle.dense(layers, x, ws)
    assert np.max(np.abs(out - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_against_torch_int_exact():
    w = wl_mod.make(4, streams=1, size=32, channels=(4, 4, 8, 8, 8, 8, 8, 8))
    x = w["x"][0]
    ref = torch_dense(w["layers"], x, w["weights"], w["biases"])
    out, per_layer = oracle.dense(w["layers"], x, w["weights"], integer=True, return_layers=True)
    assert np.array_equal(out, ref.astype(np.int64))
    assert out.max() > 0
    # every pre-activation is far from overflowing 32 bits: |c| <= 9*64*15*8
    assert max(int(np.abs(a).max()) for a in per_layer) <= 69120


def test_composition_of_two_linear_1d_convs_is_one_conv():
    # (x ⋆ a) ⋆ b = x ⋆ (a * b): correlation twice = correlation with the convolved kernels
    rng = np.random.default_rng(7)
    a, b = rng.normal(size=3), rng.normal(size=4)
    x = rng.normal(size=(40, 1, 1))
    two = oracle.dense([conv(1, 1, 3, 1, act="none"), conv(1, 1, 4, 1, act="none")], x,
                       [a.reshape(1, 1, 3, 1), b.reshape(1, 1, 4, 1)])
    ab = np.convolve(a, b)
    one = oracle.dense([conv(1, 1, 6, 1, act="none")], x, [ab.reshape(1, 1, 6, 1)])
    assert np.allclose(two, one, rtol=0, atol=1e-12)
    assert np.allclose(one.reshape(-1), np.correlate(x.reshape(-1), ab, mode="valid"), atol=1e-12)


def test_linear_superposition():
    rng = np.random.default_rng(8)
    layers = [conv(2, 3, 3, 3, p_h=1, p_w=1, act="none"), conv(3, 2, 3, 3, s=2, act="none")]
    ws = [rng.normal(size=(3, 2, 3, 3)), rng.normal(size=(2, 3, 3, 3))]
    x1, x2 = rng.normal(size=(9, 8, 2)), rng.normal(size=(9, 8, 2))
    s = oracle.dense(layers, x1 + x2, ws)
    assert np.allclose(s, oracle.dense(layers, x1, ws) + oracle.dense(layers, x2, ws), atol=1e-12)


def test_impulse_reaches_exactly_its_cone():
    # all-positive weights, identity activation: an impulse lights up a window of
    # side 1 + n(K-1) at depth n, nothing outside it (stride 1, same padding)
    rng = np.random.default_rng(9)
    layers = [conv(1, 2, 3, 3, p_h=1, p_w=1, act="none"), conv(2, 2, 3, 3, p_h=1, p_w=1, act="none"),
              conv(2, 1, 3, 3, p_h=1, p_w=1, act="none")]
    ws = [rng.random(size=(L["c_out"], L["c_in"], 3, 3)) + 0.1 for L in layers]
    x = np.zeros((21, 21, 1)); x[10, 9, 0] = 1.0
    _, per_layer = oracle.dense(layers, x, ws, return_layers=True)
    for n, a in enumerate(per_layer, start=1):
        nz = np.argwhere(np.abs(a).sum(axis=2) > 0)
        assert nz[:, 0].min() == 10 - n and nz[:, 0].max() == 10 + n
        assert nz[:, 1].min() == 9 - n and nz[:, 1].max() == 9 + n
        assert len(nz) == (1 + 2 * n) ** 2


def test_requant_commutes_with_max():
    v = np.arange(-50, 400)
    q = lambda c: np.minimum(15, np.maximum(c, 0) >> 4)
    a, b = np.meshgrid(v, v)
    assert np.array_equal(q(np.maximum(a, b)), np.maximum(q(a), q(b)))


def test_round_bf16_matches_torch_and_generator():
    rng = np.random.default_rng(11)
    vals = np.concatenate([rng.normal(size=2000) * 10.0 ** rng.integers(-6, 6, size=2000),
                           [0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e-39, 65280.0, 255.5, 256.5 * 2]])
    vals = vals.astype(np.float32)
    ref = torch.from_numpy(vals).to(torch.bfloat16).to(torch.float32).numpy()
    mine = np.array([oracle.round_bf16(float(v)) for v in vals], dtype=np.float64)
    assert np.array_equal(mine, ref.astype(np.float64))
    assert np.array_equal(wl_mod.round_to_bf16(vals), ref)
    # ties go to the even neighbour: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_bf16(1.00390625) == 1.0
    assert oracle.round_bf16(1.01171875) == 1.015625
    # a double just above a tie must round up although float32 would first land on the tie
    assert oracle.round_bf16(1.00390625 + 1e-12) == 1.0078125


def test_head_units_hand_worked():
    """Fully connected output units (Sec. 4: the class units that settle as rows come in; the
    weighted sum is the first equation of Sec. 3).  Two units over a 2x2x2 map, every weight
    distinct per (unit, row, x, c), expected values written out by hand.

    map  h[row][x][c]:  row 0: (1,2) (3,4)   row 1: (5,6) (7,8)
    unit 0 weights:     row 0: (1,10) (100,1000)   row 1: (2,20) (200,2000)
    unit 1 weights:     row 0: (-1,0) (0,1)        row 1: (3,0) (0,-2)
    bias: (0.5, -0.25)

    after row 0 only: u0 = 1*1 + 10*2 + 100*3 + 1000*4 = 4321 ; u1 = -1 + 4 = 3
    after both rows:  u0 = 4321 + 2*5 + 20*6 + 200*7 + 2000*8 = 21851 ; u1 = 3 + 15 - 16 = 2
    """
    h = np.array([[[1, 2], [3, 4]], [[5, 6], [7, 8]]], dtype=np.float64)
    w = np.array([[[[1, 10], [100, 1000]], [[2, 20], [200, 2000]]],
                  [[[-1, 0], [0, 1]], [[3, 0], [0, -2]]]], dtype=np.float64)
    b = np.array([0.5, -0.25])
    assert oracle.head_units(h[:0], w, b).tolist() == [0.5, -0.25]          # nothing arrived: the bias alone
    assert oracle.head_units(h[:1], w, b).tolist() == [4321.5, 2.75]
    assert oracle.head_units(h, w, b).tolist() == [21851.5, 1.75]
    assert oracle.head_units(h[:1], w).tolist() == [4321.0, 3.0]            # no bias
    # a transposed (x, c) or (row, x) axis gives other numbers: swap the map's axes and the result must change
    assert oracle.head_units(np.swapaxes(h, 1, 2), w).tolist() != [21851.0, 2.0]
    assert oracle.head_units(np.swapaxes(h, 0, 1), w).tolist() != [21851.0, 2.0]
    # after the last row it is the conventional network's dense layer: torch's linear on the flattened map
    full = F.linear(torch.from_numpy(h.reshape(1, -1)), torch.from_numpy(w.reshape(2, -1)), torch.from_numpy(b))
    assert np.array_equal(oracle.head_units(h, w, b), full[0].numpy())
