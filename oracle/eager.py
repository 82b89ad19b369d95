"""Paper-literal eager event scheme (tiny nets only).  TEST INFRASTRUCTURE ONLY.

Every neuron of every layer exists for the whole sample and follows Sec. 3 to
the letter: it keeps its state variable c, and whenever f(c) differs from the
value it last announced it emits the difference as an event at once; the event
is added, weighted, into the c of each neuron it connects to, which may in turn
emit.  Nothing is ever forgotten here and nothing waits for a row to complete,
so after *any* prefix of the input the announced activations of every layer
equal the conventional network applied to the input seen so far (the rest
taken as zero) -- the equality the paper states just after its event-delivery
rule and draws in Fig. 3 (accumulated output over the 28 row presentations).

Pure Python loops over numpy arrays; independent of idfo.c on purpose.
"""
from __future__ import annotations

import numpy as np


def _act(L, c):
    a = L.get("act", "none")
    if a == "none":
        return c
    if a == "relu":
        return c if c > 0 else c * 0
    if a == "relu_shr_clamp":
        r = c if c > 0 else c * 0
        r = int(r) >> L["shr"]
        return min(r, L["clamp_hi"])
    raise ValueError(a)


def _out_size(n, k, s, p):
    t = n + 2 * p - k
    return 0 if t < 0 else t // s + 1


class EagerNet:
    def __init__(self, layers, in_h, in_w, in_c, weights, biases=None, dtype=np.float64):
        self.layers = layers
        self.dtype = dtype
        self.w = [None if w is None else np.asarray(w, dtype=dtype) for w in weights]
        biases = biases if biases is not None else [None] * len(layers)
        self.shapes = [(in_h, in_w, in_c)]
        for L in layers:
            h, w, _ = self.shapes[-1]
            self.shapes.append((_out_size(h, L["k_h"], L["s_h"], L["p_h"]),
                                _out_size(w, L["k_w"], L["s_w"], L["p_w"]), L["c_out"]))
        # announced[n]: value each neuron of layer n last announced (layer 0 = input)
        self.announced = [np.zeros(s, dtype=dtype) for s in self.shapes]
        # c[n]: state variable of conv layer n+1's neurons; for a pool node the
        # current values of its inputs (max is not additive, it is re-evaluated)
        self.c = [np.zeros(self.shapes[i + 1] if L["kind"] == "conv" else self.shapes[i], dtype=dtype)
                  for i, L in enumerate(layers)]
        self.events = [0] * (len(layers) + 1)      # events emitted by layer n (0 = input)
        # a bias is a constant input present from the start: one initial event per neuron
        for n, L in enumerate(layers):
            b = biases[n]
            if L["kind"] == "conv" and b is not None:
                H, W, Cc = self.shapes[n + 1]
                for y in range(H):
                    for x in range(W):
                        for co in range(Cc):
                            self.c[n][y, x, co] += dtype(b[co])
                            self._reconsider(n, y, x, co)

    # neuron (y,x,co) of layer n+1 had its state changed: announce a change, if any
    def _reconsider(self, n, y, x, co):
        L = self.layers[n]
        new = _act(L, self.c[n][y, x, co])
        d = new - self.announced[n + 1][y, x, co]
        if d != 0:
            self.announced[n + 1][y, x, co] = new
            self._emit(n + 1, y, x, co, d)

    # neuron (y,x,ch) of layer `src` (0 = input) announces change d
    def _emit(self, src, y, x, ch, d):
        self.events[src] += 1
        if src == len(self.layers):
            return
        L = self.layers[src]
        H_o, W_o, C_o = self.shapes[src + 1]
        if L["kind"] == "conv":
            w = self.w[src]
            for ky in range(L["k_h"]):
                t = y + L["p_h"] - ky
                if t < 0 or t % L["s_h"] or t // L["s_h"] >= H_o:
                    continue
                for kx in range(L["k_w"]):
                    u = x + L["p_w"] - kx
                    if u < 0 or u % L["s_w"] or u // L["s_w"] >= W_o:
                        continue
                    oy, ox = t // L["s_h"], u // L["s_w"]
                    for co in range(C_o):
                        self.c[src][oy, ox, co] += w[co, ch, ky, kx] * d
                        self._reconsider(src, oy, ox, co)
        else:  # stateful max node
            self.c[src][y, x, ch] += d
            oy, ox = y // 2, x // L["s_w"]
            if oy >= H_o or ox >= W_o:
                return
            win = self.c[src][2 * oy:2 * oy + 2, ox * L["s_w"]:ox * L["s_w"] + L["k_w"], ch]
            new = win.max()
            dd = new - self.announced[src + 1][oy, ox, ch]
            if dd != 0:
                self.announced[src + 1][oy, ox, ch] = new
                self._emit(src + 1, oy, ox, ch, dd)

    def present(self, y, x, ch, value):
        """One input component arrives (its previous value was zero)."""
        d = self.dtype(value) - self.announced[0][y, x, ch]
        if d != 0:
            self.announced[0][y, x, ch] = self.dtype(value)
            self._emit(0, y, x, ch, d)

    def present_row(self, y, row):
        row = np.asarray(row)
        for x in range(row.shape[0]):
            for ch in range(row.shape[1]):
                self.present(y, x, ch, row[x, ch])
