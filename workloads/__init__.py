"""Seeded synthetic workloads: network descriptions, weights and input streams.

This module only *generates arrays*.  It contains none of the method's
arithmetic (no convolution, no activation, no event logic) so that it can feed
both the CPU oracle and the GPU library without making them share code.  A
workload is a plain dict:

    name        str
    precision   'f32' | 'bf16' | 'i8'
    in_h        rows per sample (0 would mean unbounded; every config is bounded)
    in_w, in_c  row width and channels (1-D signals: in_w = 1)
    layers      list of dicts: kind ('conv'|'maxpool'), c_in, c_out, k_h, k_w,
                s_h, s_w, p_h, p_w, act ('none'|'relu'|'relu_shr_clamp'), shr, clamp_hi
    weights     per layer: None (pool) or array [C_out][C_in][K_h][K_w]
                (float32; bf16 workloads hold bf16-representable float32; i8: int8)
    biases      per layer: None or array [C_out] (float32 / int32)
    x           input, [streams][in_h][in_w][in_c] (float32, bf16-representable
                float32, or int8)
    seg_rows    rows handed over per push in the stated workload
    streams     number of independent streams

The five configurations are those the build is measured on; none of them is a
published dataset -- they stand in, with the same structure (rows arriving one
at a time, large all-zero regions), for the image data the paper used.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 180410727 * 10


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return (u.astype(np.uint32) << 16).view(np.float32).reshape(a.shape)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Bit patterns (uint16) of bf16-representable float32 values."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(a.shape)


def conv(c_in, c_out, k_h, k_w, s=1, p_h=0, p_w=0, act="relu", shr=0, clamp_hi=0):
    return dict(kind="conv", c_in=c_in, c_out=c_out, k_h=k_h, k_w=k_w, s_h=s,
                s_w=(s if k_w > 1 else 1), p_h=p_h, p_w=p_w, act=act, shr=shr, clamp_hi=clamp_hi)


def maxpool(c, k_w=2):
    return dict(kind="maxpool", c_in=c, c_out=c, k_h=2, k_w=k_w, s_h=2, s_w=k_w,
                p_h=0, p_w=0, act="none", shr=0, clamp_hi=0)


def out_size(n, k, s, p):
    t = n + 2 * p - k
    return 0 if t < 0 else t // s + 1


def output_shape(wl):
    """(rows, width, channels) of the last layer's output for one sample."""
    h, w, c = wl["in_h"], wl["in_w"], wl["in_c"]
    for L in wl["layers"]:
        h = out_size(h, L["k_h"], L["s_h"], L["p_h"])
        w = out_size(w, L["k_w"], L["s_w"], L["p_w"])
        c = L["c_out"]
    return h, w, c


def dense_equivalent_macs_by_layer(wl):
    """Multiply-adds of the conventional network for one sample, layer by layer (0 for pools), padding taps included."""
    h, w = wl["in_h"], wl["in_w"]
    per = []
    for L in wl["layers"]:
        h = out_size(h, L["k_h"], L["s_h"], L["p_h"])
        w = out_size(w, L["k_w"], L["s_w"], L["p_w"])
        per.append(h * w * L["k_h"] * L["k_w"] * L["c_in"] * L["c_out"] if L["kind"] == "conv" else 0)
    return per


def dense_equivalent_macs(wl):
    """Multiply-adds of the conventional network for one sample, padding taps included."""
    return sum(dense_equivalent_macs_by_layer(wl))


def _normal_weights(rng, layers, var_num, dtype=np.float32):
    ws = []
    for L in layers:
        if L["kind"] != "conv":
            ws.append(None)
            continue
        fan_in = L["c_in"] * L["k_h"] * L["k_w"]
        w = rng.normal(0.0, np.sqrt(var_num / fan_in),
                       size=(L["c_out"], L["c_in"], L["k_h"], L["k_w"]))
        ws.append(w.astype(dtype))
    return ws


def _finish(name, precision, in_h, in_w, in_c, layers, weights, biases, x, seg_rows):
    return dict(name=name, precision=precision, in_h=in_h, in_w=in_w, in_c=in_c,
                layers=layers, weights=weights, biases=biases, x=x,
                seg_rows=seg_rows, streams=x.shape[0])


def cfg1(streams=1, length=4096, seed=SEED_BASE + 1):
    """1-D, 3 conv layers K=3 valid, 1->8->8->8, ReLU, with biases; one sample per push."""
    rng = np.random.default_rng(seed)
    x = rng.random((streams, length, 1, 1)).astype(np.float32)
    x[rng.random(x.shape) < 0.5] = 0.0
    layers = [conv(1, 8, 3, 1), conv(8, 8, 3, 1), conv(8, 8, 3, 1)]
    weights = _normal_weights(rng, layers, 1.0)
    biases = [rng.normal(0.0, 0.1, size=(L["c_out"],)).astype(np.float32) for L in layers]
    return _finish("cfg1_1d_k3", "f32", length, 1, 1, layers, weights, biases, x, 1)


def cfg2(streams=64, length=16000, seed=SEED_BASE + 2, channels=(32, 32, 64, 64, 64, 64)):
    """1-D audio-like, 6 conv layers K=9 valid, stride 2 on conv 2 and 4; 16 samples per push."""
    rng = np.random.default_rng(seed)
    x = rng.normal(0.0, 1.0, size=(streams, length, 1, 1)).astype(np.float32)
    for b in range(streams):
        zero = np.zeros(length, dtype=bool)
        while zero.mean() < 0.4:
            n = int(rng.integers(10, 201))
            s = int(rng.integers(0, length))
            zero[s:s + n] = True
        x[b, zero, 0, 0] = 0.0
    chans = (1,) + tuple(channels)
    layers = [conv(chans[i], chans[i + 1], 9, 1, s=(2 if i in (1, 3) else 1)) for i in range(6)]
    weights = _normal_weights(rng, layers, 2.0)
    biases = [None] * len(layers)
    return _finish("cfg2_1d_audio_k9", "f32", length, 1, 1, layers, weights, biases, x, 16)


def cfg3(streams=256, size=32, seed=SEED_BASE + 3, channels=(32, 32, 64, 64)):
    """2-D small CNN: c3x3, c3x3, pool, c3x3, c3x3, same padding, ReLU; one row per push."""
    rng = np.random.default_rng(seed)
    x = rng.random((streams, size, size, 3)).astype(np.float32)
    x[rng.random((streams, size, size)) < 0.6] = 0.0
    c = channels
    layers = [conv(3, c[0], 3, 3, p_h=1, p_w=1), conv(c[0], c[1], 3, 3, p_h=1, p_w=1), maxpool(c[1]),
              conv(c[1], c[2], 3, 3, p_h=1, p_w=1), conv(c[2], c[3], 3, 3, p_h=1, p_w=1)]
    weights = _normal_weights(rng, layers, 2.0)
    biases = [None] * len(layers)
    return _finish("cfg3_2d_small", "f32", size, size, 3, layers, weights, biases, x, 1)


def cfg4(streams=32, size=224, seed=SEED_BASE + 4, channels=(16, 16, 32, 32, 64, 64, 64, 64)):
    """2-D quantised event CNN: int8 input in {0..15} in blobs, 8 conv3x3 same, pool after
    conv 2, 4, 6; ReLU, >>4, clamp to [0,15] between layers; last layer plain ReLU (int32)."""
    rng = np.random.default_rng(seed)
    x = np.zeros((streams, size, size, 1), dtype=np.int8)
    yy, xx = np.mgrid[0:size, 0:size]
    for b in range(streams):
        img = x[b, :, :, 0]
        while np.count_nonzero(img) < 0.2 * size * size:
            cy, cx = rng.integers(0, size, size=2)
            r = int(rng.integers(3, 17))
            disc = (yy - cy) ** 2 + (xx - cx) ** 2 <= r * r
            vals = rng.integers(1, 16, size=(size, size)).astype(np.int8)
            img[disc] = vals[disc]
    chans = (1,) + tuple(channels)
    layers = []
    for i in range(8):
        last = i == 7
        layers.append(conv(chans[i], chans[i + 1], 3, 3, p_h=1, p_w=1,
                           act=("relu" if last else "relu_shr_clamp"),
                           shr=(0 if last else 4), clamp_hi=(0 if last else 15)))
        if i in (1, 3, 5):
            layers.append(maxpool(chans[i + 1]))
    weights = [None if L["kind"] != "conv" else
               rng.integers(-8, 8, size=(L["c_out"], L["c_in"], 3, 3)).astype(np.int8) for L in layers]
    biases = [None] * len(layers)
    return _finish("cfg4_2d_int8_events", "i8", size, size, 1, layers, weights, biases, x, 1)


def cfg5(streams=64, size=224, seed=SEED_BASE + 5, channels=(64, 64, 128, 128, 256, 256, 256)):
    """2-D VGG-style front in bf16 with fp32 state: c,c,pool,c,c,pool,c,c,c; one row per push."""
    rng = np.random.default_rng(seed)
    x = rng.random((streams, size, size, 3), dtype=np.float32)
    x[rng.random((streams, size, size)) < 0.3] = 0.0
    x = round_to_bf16(x)
    c = channels
    layers = [conv(3, c[0], 3, 3, p_h=1, p_w=1), conv(c[0], c[1], 3, 3, p_h=1, p_w=1), maxpool(c[1]),
              conv(c[1], c[2], 3, 3, p_h=1, p_w=1), conv(c[2], c[3], 3, 3, p_h=1, p_w=1), maxpool(c[3]),
              conv(c[3], c[4], 3, 3, p_h=1, p_w=1), conv(c[4], c[5], 3, 3, p_h=1, p_w=1),
              conv(c[5], c[6], 3, 3, p_h=1, p_w=1)]
    weights = [None if w is None else round_to_bf16(w) for w in _normal_weights(rng, layers, 2.0)]
    biases = [None] * len(layers)
    return _finish("cfg5_2d_vgg_bf16", "bf16", size, size, 3, layers, weights, biases, x, 1)


CONFIGS = {1: cfg1, 2: cfg2, 3: cfg3, 4: cfg4, 5: cfg5}


def make(cfg: int, **kw):
    """Workload `cfg` (1..5) at its stated size, or scaled down through keyword arguments."""
    return CONFIGS[cfg](**kw)
