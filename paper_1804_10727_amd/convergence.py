"""Accumulated output against rows presented (Sec. 4, the experiment behind Fig. 3 and Fig. 4): class
units over the last layer's map, read after every pushed row.  After the last row their values are
those of the conventional network; the curve shows how early they settle.

The paper's curve is for a trained MNIST classifier; neither the data nor the weights exist here, so
this runs the same measurement on a synthetic workload with random class-unit weights: what it shows
is the mechanics (values converge monotonically in coverage, exactly at the last row), not accuracy.

    python -m paper_1804_10727_amd.convergence [--config 3] [--units 10] [--streams 256]
"""
from __future__ import annotations

import argparse

import numpy as np


def curve(wl, n_units=10, seed=9):
    """Pushes every stream's sample one row at a time and reads the class units after every row.

    Returns (rows_seen [H], values [H][streams][units], unit_weights, unit_bias): values[r] are
    the units after input row r; rows_seen[r] the output rows accumulated by then."""
    from . import net_from_workload, Streams
    from .binding import input_tensor
    B, H = wl["streams"], wl["in_h"]
    net = net_from_workload(wl)
    st = Streams(net, B, max_seg_rows=1)
    oh, ow, oc = int(st.sizes.out_h), int(st.sizes.out_w), int(st.sizes.out_c)
    rng = np.random.default_rng(seed)
    w = rng.normal(0, 1.0 / np.sqrt(oh * ow * oc), size=(n_units, oh, ow, oc)).astype(np.float32)
    b = rng.normal(0, 0.1, size=(n_units,)).astype(np.float32)
    st.enable_head_units(w, b)
    x = input_tensor(wl)
    vals = np.zeros((H, B, n_units))
    seen = np.zeros(H, dtype=np.int64)
    for r in range(H):
        st.push_segment(x[:, r:r + 1].contiguous())
        rows, v = st.read_head_units()
        vals[r] = v
        seen[r] = rows[0]
    st.close()
    net.destroy()
    return seen, vals, w, b


def summarise(seen, vals):
    """Per input row: output rows accumulated, share of samples whose largest unit is already the
    final one, and the mean distance to the final values relative to their spread."""
    final = vals[-1]
    scale = max(float(np.std(final)), 1e-30)
    win = np.argmax(final, axis=1)
    out = []
    for r in range(vals.shape[0]):
        out.append((r + 1, int(seen[r]), float(np.mean(np.argmax(vals[r], axis=1) == win)),
                    float(np.mean(np.abs(vals[r] - final)) / scale)))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--units", type=int, default=10)
    ap.add_argument("--streams", type=int, default=None)
    args = ap.parse_args()
    import workloads
    kw = {} if args.streams is None else {"streams": args.streams}
    wl = workloads.make(args.config, **kw)
    seen, vals, _, _ = curve(wl, args.units)
    print(f"workload {wl['name']}, {wl['streams']} samples, {args.units} class units with random weights")
    print("| input rows presented | output rows accumulated | samples whose largest unit is the final one | mean distance to final values / their std |")
    print("|---|---|---|---|")
    rows = summarise(seen, vals)
    step = max(1, len(rows) // 16)
    for i, (r, s, agree, dist) in enumerate(rows):
        if i % step == step - 1 or i == len(rows) - 1 or i == 0:
            print(f"| {r} | {s} | {agree:.3f} | {dist:.4f} |")


if __name__ == "__main__":
    main()
