"""Pins of the volume oracle (oracle/volume.py): inputs of more than two dimensions, which Sec. 3
names as a further case of the same scheme.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import volume as V
import oracle


def _net(rng, chans, ks, ss, ps, acts, integer=False):
    layers, weights = [], []
    for i in range(len(chans) - 1):
        layers.append(dict(c_in=chans[i], c_out=chans[i + 1], k=ks[i], s=ss[i], p=ps[i], act=acts[i], shr=2, clamp_hi=15))
        shape = (chans[i + 1], chans[i]) + tuple(ks[i])
        weights.append(rng.integers(-3, 4, size=shape).astype(np.float64) if integer else rng.normal(size=shape))
    return layers, weights


def test_dense3d_hand_worked():
    # one layer, 1 -> 1 channel, kernel 2x2x2 of weights 1..8 (slab-major), no padding, on a 2x2x3 volume:
    # out[0,0,w] = sum_{a,b,e} w[a][b][e] * x[a][b][w+e]
    x = np.arange(1, 13, dtype=np.float64).reshape(2, 2, 3, 1)          # x[d][h][w] = 1 + 6d + 3h + w
    w = np.arange(1, 9, dtype=np.float64).reshape(1, 1, 2, 2, 2)
    L = [dict(c_in=1, c_out=1, k=(2, 2, 2), s=(1, 1, 1), p=(0, 0, 0), act="none")]
    out = V.dense3d(L, x, [w])
    # w = [[[1,2],[3,4]],[[5,6],[7,8]]]; at ow=0 the window is x[d][h][0..1] = {1,2 | 4,5 || 7,8 | 10,11}
    e0 = 1 * 1 + 2 * 2 + 3 * 4 + 4 * 5 + 5 * 7 + 6 * 8 + 7 * 10 + 8 * 11
    e1 = 1 * 2 + 2 * 3 + 3 * 5 + 4 * 6 + 5 * 8 + 6 * 9 + 7 * 11 + 8 * 12
    assert out.shape == (1, 1, 2, 1)
    assert out[0, 0, 0, 0] == e0 == 278 and out[0, 0, 1, 0] == e1 == 314


def test_dense3d_padding_and_stride_hand_worked():
    # an impulse of 2 at (1,0,2) through a 3x3x3 kernel, padding 1, stride (1,2,1): the output at (od,oh,ow)
    # is 2 * w[1-od+1][0-2oh+1][2-ow+1] where those are taps
    x = np.zeros((3, 3, 4, 1)); x[1, 0, 2, 0] = 2.0
    w = np.arange(27, dtype=np.float64).reshape(1, 1, 3, 3, 3)
    L = [dict(c_in=1, c_out=1, k=(3, 3, 3), s=(1, 2, 1), p=(1, 1, 1), act="none")]
    out = V.dense3d(L, x, [w])
    assert out.shape == (3, 2, 4, 1)
    exp = np.zeros((3, 2, 4))
    for od in range(3):
        for oh in range(2):
            for ow in range(4):
                a, b, e = 1 - od + 1, 0 - 2 * oh + 1, 2 - ow + 1
                if 0 <= a < 3 and 0 <= b < 3 and 0 <= e < 3:
                    exp[od, oh, ow] = 2.0 * (9 * a + 3 * b + e)
    assert exp[1, 0, 2] == 2.0 * 13 and exp[0, 0, 3] == 2.0 * (18 + 3 + 0)        # spot values by hand
    assert np.array_equal(out[..., 0], exp)


@pytest.mark.parametrize("seed,ks,ss,ps", [
    (0, [(3, 3, 3), (3, 3, 3)], [(1, 1, 1), (1, 1, 1)], [(1, 1, 1), (1, 1, 1)]),
    (1, [(2, 3, 1), (3, 1, 2)], [(1, 2, 1), (2, 1, 1)], [(0, 1, 0), (1, 0, 1)]),
    (2, [(3, 3, 3), (1, 1, 1), (2, 2, 2)], [(2, 1, 1), (1, 1, 1), (1, 1, 2)], [(1, 0, 1), (0, 0, 0), (0, 1, 0)]),
])
def test_dense3d_against_library_convolution(seed, ks, ss, ps):
    rng = np.random.default_rng(seed)
    chans = [2, 3, 4, 2][:len(ks) + 1]
    layers, weights = _net(rng, chans, ks, ss, ps, ["relu"] * (len(ks) - 1) + ["none"])
    biases = [rng.normal(size=c) for c in chans[1:]]
    x = rng.normal(size=(7, 6, 5, chans[0])) * (rng.random((7, 6, 5, 1)) < 0.6)
    out = V.dense3d(layers, x, weights, biases)
    h = torch.tensor(x, dtype=torch.float64).permute(3, 0, 1, 2)[None]
    for i, L in enumerate(layers):
        h = torch.nn.functional.conv3d(h, torch.tensor(weights[i]), torch.tensor(biases[i]), stride=L["s"], padding=L["p"])
        if L["act"] == "relu":
            h = torch.relu(h)
    ref = h[0].permute(1, 2, 3, 0).numpy()
    assert out.shape == ref.shape
    assert np.abs(out - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())


@pytest.mark.parametrize("seg", [1, 2, 3, 7])
@pytest.mark.parametrize("seed,ks,ss,ps", [
    (3, [(3, 3, 3), (3, 3, 3)], [(1, 1, 1), (1, 1, 1)], [(1, 1, 1), (1, 1, 1)]),
    (4, [(2, 3, 1), (3, 1, 2)], [(1, 2, 1), (2, 1, 1)], [(0, 1, 0), (1, 0, 1)]),
    (5, [(3, 2, 2), (3, 3, 3)], [(2, 1, 1), (1, 1, 1)], [(1, 0, 0), (0, 1, 1)]),
])
def test_streamed_equals_dense_for_any_segmenting(seed, ks, ss, ps, seg):
    rng = np.random.default_rng(seed)
    layers, weights = _net(rng, [2, 3, 2], ks, ss, ps, ["relu", "relu"], integer=True)
    biases = [rng.integers(-2, 3, size=c) for c in (3, 2)]
    x = rng.integers(-4, 5, size=(7, 5, 6, 2)) * (rng.random((7, 5, 6, 1)) < 0.5)
    ref = V.dense3d(layers, x, weights, biases, integer=True)
    out, st = V.stream3d_run(layers, x, weights, biases, seg=seg, integer=True)
    assert np.array_equal(out, ref)
    # a layer never holds more slabs than its kernel is deep, whatever the number of slabs
    for L, peak in zip(layers, st["peak_slabs"]):
        assert peak <= L["k"][0]


def test_live_slabs_do_not_grow_with_depth_of_the_volume():
    rng = np.random.default_rng(6)
    layers, weights = _net(rng, [1, 2, 2], [(3, 3, 3)] * 2, [(1, 1, 1)] * 2, [(1, 1, 1)] * 2, ["relu", "relu"])
    peaks = []
    for D in (5, 9, 14):
        x = rng.random((D, 4, 4, 1))
        _, st = V.stream3d_run(layers, x, weights)
        peaks.append(tuple(st["peak_slabs"]))
    assert peaks[0] == peaks[1] == peaks[2] == (3, 3)


def test_zero_volume_gives_no_events_and_counts_match_brute_force():
    rng = np.random.default_rng(7)
    layers, weights = _net(rng, [2, 3], [(3, 2, 3)], [(1, 1, 2)], [(1, 0, 1)], ["relu"])
    z = np.zeros((4, 3, 5, 2))
    out, st = V.stream3d_run(layers, z, weights)
    assert st["events_in"].sum() == 0 and st["macs"].sum() == 0 and not out.any()
    x = rng.normal(size=(4, 3, 5, 2)) * (rng.random((4, 3, 5, 2)) < 0.4)
    _, st = V.stream3d_run(layers, x, weights)
    L = layers[0]
    Do, Ho, Wo, Co = V.shapes3d(layers, 4, 3, 5)[0]
    macs = 0
    for zd, zh, zw, _ in zip(*np.nonzero(x)):
        for od in range(Do):
            for oh in range(Ho):
                for ow in range(Wo):
                    a, b, e = zd - (od * 1 - 1), zh - (oh * 1 - 0), zw - (ow * 2 - 1)
                    if 0 <= a < 3 and 0 <= b < 2 and 0 <= e < 3:
                        macs += Co
    assert st["events_in"][0] == np.count_nonzero(x) and st["macs"][0] == macs


def test_a_volume_one_column_wide_is_the_image_case():
    # a volume [D][H][1][C] with kernels 1 wide is an image [D][H][C]: both oracles must agree
    rng = np.random.default_rng(8)
    w3 = [rng.normal(size=(3, 2, 3, 3, 1)), rng.normal(size=(2, 3, 3, 3, 1))]
    L3 = [dict(c_in=2, c_out=3, k=(3, 3, 1), s=(1, 1, 1), p=(1, 1, 0), act="relu"),
          dict(c_in=3, c_out=2, k=(3, 3, 1), s=(1, 1, 1), p=(1, 1, 0), act="relu")]
    L2 = [dict(kind="conv", c_in=2, c_out=3, k_h=3, k_w=3, s_h=1, s_w=1, p_h=1, p_w=1, act="relu"),
          dict(kind="conv", c_in=3, c_out=2, k_h=3, k_w=3, s_h=1, s_w=1, p_h=1, p_w=1, act="relu")]
    x = rng.normal(size=(6, 5, 1, 2))
    a = V.dense3d(L3, x, w3)
    b = oracle.dense(L2, x[:, :, 0, :], [w[..., 0] for w in w3])
    assert np.abs(a[:, :, 0, :] - b).max() <= 1e-12


def test_round_bf16_matches_library_rounding():
    rng = np.random.default_rng(9)
    v = np.concatenate([rng.normal(size=2000) * 10.0 ** rng.integers(-3, 4, size=2000),
                        [1.00390625, 1.01171875, 1.0 + 2.0 ** -8 + 2.0 ** -30, 0.0]])   # ties (to even) and just above a tie
    ref = torch.tensor(v, dtype=torch.float64).to(torch.float32)
    # float64 -> float32 is exact for these checks only where no double rounding can occur: compare on values
    # that are float32 already
    v32 = ref.to(torch.float64).numpy()
    got = V.round_bf16(v32)
    exp = ref.to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, exp)
    assert V.round_bf16(1.0 + 2.0 ** -8 + 2.0 ** -30) == 1.0 + 2.0 ** -7      # a double just above a tie rounds up
