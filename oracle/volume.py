"""Oracle for volumes presented slab by slab.  TEST INFRASTRUCTURE ONLY.

Sec. 3 remarks that the scheme carries over to inputs of more than two
dimensions; for a volume [slab][row][column][channel] that arrives one slab at
a time this file holds

  * ``dense3d``: the conventional network, one whole layer after another, each
    a direct convolution written out over output position and tap (first
    equation of Sec. 3 with three spatial indices), float64 or int64;
  * ``Stream3d``: the paper's scheme along the slab axis -- every non-zero
    value of an arriving slab is one event that is added, weighted, into the
    state c of each neuron it connects to (event-delivery rule of Sec. 3); a
    layer keeps a rolling buffer of k_d slabs of c; a slab of c is activated,
    handed on (depth-first) and forgotten when the last input slab its
    definition needs has arrived.  Counts events, multiply-adds and the slabs
    alive at once.

Pure Python loops over numpy arrays, for small volumes; independent of idfo.c
and of the GPU library on purpose.  Layers are dicts with c_in, c_out, k, s, p
(triples over slab, row, column), act ('none' | 'relu' | 'relu_shr_clamp'),
shr, clamp_hi; weights [c_out][c_in][k_d][k_h][k_w].

Parity status: pinned by tests/test_oracle_volume.py (hand-worked values, a
library 3-D convolution in float64, dense == streamed for every segmenting,
the bound of k_d live slabs, counts by brute force).
"""
from __future__ import annotations

import numpy as np


def out_size(n, k, s, p):
    t = n + 2 * p - k
    return 0 if t < 0 else t // s + 1


def round_bf16(a):
    """Round float64 values to the nearest bfloat16 value (8 significant bits, ties to even), as float64.
    Written for the normal range: a = m * 2**e with 0.5 <= |m| < 1 is rounded at the eighth bit of m."""
    a = np.asarray(a, dtype=np.float64)
    m, e = np.frexp(a)
    return np.ldexp(np.rint(m * 256.0), e - 8)


def activate(L, c, integer):
    a = L.get("act", "none")
    if a == "none":
        return c
    r = np.maximum(c, 0)
    if a == "relu":
        return r
    if a == "relu_shr_clamp":
        assert integer
        return np.minimum(r >> L["shr"], L["clamp_hi"])
    raise ValueError(a)


def shapes3d(layers, in_d, in_h, in_w):
    out = []
    d, h, w = in_d, in_h, in_w
    for L in layers:
        d, h, w = (out_size(n, k, s, p) for n, k, s, p in zip((d, h, w), L["k"], L["s"], L["p"]))
        out.append((d, h, w, L["c_out"]))
    return out


def dense3d(layers, x, weights, biases=None, *, integer=False, emit_round=None, return_layers=False):
    """The conventional 3-D network on one sample x [D][H][W][C0]."""
    dt = np.int64 if integer else np.float64
    h = np.asarray(x, dtype=dt)
    outs = []
    for li, L in enumerate(layers):
        w = np.asarray(weights[li], dtype=dt)                   # [co][ci][kd][kh][kw]
        D, H, W, C = h.shape
        assert C == L["c_in"]
        (kd, kh, kw), (sd, sh, sw), (pd, ph, pw) = L["k"], L["s"], L["p"]
        Do, Ho, Wo = out_size(D, kd, sd, pd), out_size(H, kh, sh, ph), out_size(W, kw, sw, pw)
        c = np.zeros((Do, Ho, Wo, L["c_out"]), dtype=dt)
        if biases is not None and biases[li] is not None:
            c += np.asarray(biases[li], dtype=dt)
        for od in range(Do):
            for oh in range(Ho):
                for ow in range(Wo):
                    for a in range(kd):
                        for b in range(kh):
                            for e in range(kw):
                                zd, zh, zw = od * sd - pd + a, oh * sh - ph + b, ow * sw - pw + e
                                if 0 <= zd < D and 0 <= zh < H and 0 <= zw < W:
                                    c[od, oh, ow] += w[:, :, a, b, e] @ h[zd, zh, zw]
        h = activate(L, c, integer)
        if emit_round == "bf16" and li < len(layers) - 1:
            h = round_bf16(h)
        outs.append(h)
    return (h, outs) if return_layers else h


class Stream3d:
    """One stream of the scheme along the slab axis: scalar events, k_d slabs of state per layer."""

    def __init__(self, layers, in_d, in_h, in_w, in_c, weights, biases=None, *, integer=False, emit_round=None):
        self.layers, self.integer, self.emit_round = layers, integer, emit_round
        self.dt = np.int64 if integer else np.float64
        self.w = [np.asarray(a, dtype=self.dt) for a in weights]
        self.b = [None if (biases is None or b is None) else np.asarray(b, dtype=self.dt)
                  for b in (biases if biases is not None else [None] * len(layers))]
        self.in_shape = [(in_d, in_h, in_w, in_c)] + shapes3d(layers, in_d, in_h, in_w)
        n = len(layers)
        self.c = [dict() for _ in range(n)]          # per layer: output slab index -> array [Ho][Wo][Co], while alive
        self.seen = [0] * n                          # input slabs the layer has received
        self.done = [0] * n                          # output slabs it has emitted
        self.events = np.zeros(n, dtype=np.int64)
        self.macs = np.zeros(n, dtype=np.int64)
        self.peak_slabs = np.zeros(n, dtype=np.int64)
        self.out = []

    def _fresh(self, li):
        _, Ho, Wo, Co = self.in_shape[li + 1]
        c = np.zeros((Ho, Wo, Co), dtype=self.dt)
        if self.b[li] is not None:
            c += self.b[li]
        return c

    def _deliver(self, li, z, slab):
        """Input slab z of layer li arrives (values [H][W][C])."""
        if li == len(self.layers):
            self.out.append(slab)
            return
        L = self.layers[li]
        D, H, W, C = self.in_shape[li]
        Do, Ho, Wo, Co = self.in_shape[li + 1]
        (kd, kh, kw), (sd, sh, sw), (pd, ph, pw) = L["k"], L["s"], L["p"]
        w = self.w[li]
        for y, x, ci in zip(*np.nonzero(slab)):
            v = slab[y, x, ci]
            self.events[li] += 1
            for a in range(kd):
                t = z + pd - a
                if t % sd or not 0 <= t // sd < Do:
                    continue
                od = t // sd
                if od not in self.c[li]:
                    self.c[li][od] = self._fresh(li)
                for b in range(kh):
                    u = y + ph - b
                    if u % sh or not 0 <= u // sh < Ho:
                        continue
                    for e in range(kw):
                        q = x + pw - e
                        if q % sw or not 0 <= q // sw < Wo:
                            continue
                        self.c[li][od][u // sh, q // sw] += v * w[:, ci, a, b, e]
                        self.macs[li] += Co
        self.peak_slabs[li] = max(self.peak_slabs[li], len(self.c[li]))
        self.seen[li] = z + 1
        # output slab o needs input slabs o*sd - pd .. o*sd - pd + kd - 1 (those that exist): final once the last has come
        while self.done[li] < Do:
            o = self.done[li]
            last_needed = min(o * sd - pd + kd - 1, D - 1)
            if last_needed > z:
                break
            c = self.c[li].pop(o, None)
            if c is None:
                c = self._fresh(li)                  # no event reached it
            hval = activate(L, c, self.integer)
            if self.emit_round == "bf16" and li < len(self.layers) - 1:
                hval = round_bf16(hval)
            self.done[li] += 1
            self._deliver(li + 1, o, hval)           # depth-first: before the next input slab is looked at

    def push(self, slabs):
        slabs = np.asarray(slabs, dtype=self.dt)
        for s in slabs:
            self._deliver(0, self.seen[0], s)

    def take(self):
        out, self.out = self.out, []
        _, Ho, Wo, Co = self.in_shape[-1]
        return np.stack(out) if out else np.empty((0, Ho, Wo, Co), dtype=self.dt)


def stream3d_run(layers, x, weights, biases=None, *, seg=1, integer=False, emit_round=None):
    D, H, W, C = x.shape
    s = Stream3d(layers, D, H, W, C, weights, biases, integer=integer, emit_round=emit_round)
    chunks = []
    for z in range(0, D, seg):
        s.push(x[z:z + seg])
        chunks.append(s.take())
    return np.concatenate(chunks, axis=0), dict(events_in=s.events, macs=s.macs, peak_slabs=s.peak_slabs)
