"""Shared by the tests: run a workload through the GPU library / through the CPU oracle."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
import workloads as wl_mod

# Tolerances (max |gpu - oracle| over one stream's output, divided by max |oracle|):
#   f32: 1e-4 (fp32 accumulation of at most 9*256 products per output against fp64)
#   bf16 against the oracle that rounds emitted activations to bf16 like the kernels: 1e-2
#        (a sum within fp32 rounding of a bf16 tie may round the other way: one bf16 ulp,
#        2^-8 relative, on single activations) and against the unrounded oracle: 2e-2
#   i8: bit exact
TOL = {"f32": 1e-4, "bf16_emul": 1e-2, "bf16_true": 2e-2}


def rel_err(g, o):
    return float(np.max(np.abs(g.astype(np.float64) - o)) / max(float(np.max(np.abs(o))), 1e-30))


# Element by element: |g - o| <= atol + rtol * |o|, with atol a small fraction of the stream's
# largest output.  A sum of n products accumulated in float32 is off by up to about
# n * 2^-24 * sum|terms| whatever its own size, so an output near zero (cancellation, or a ReLU
# about to cut) cannot be held to a purely relative bound: atol covers that floor, five times
# below the normalised tolerance for float32; rtol is the tolerance itself.  With bfloat16 events an
# activation whose float32 sum lies within rounding of a bfloat16 tie may be emitted one ulp (2^-8
# of its value) away from the oracle's, and every output it feeds moves by weight * ulp whatever
# that output's own size: atol is 2.5 times below the normalised tolerance there.
ELEM = {"f32": (2e-5, 1e-4), "bf16_emul": (4e-3, 1e-2), "bf16_true": (8e-3, 2e-2)}


def elem_excess(g, o, kind):
    """Largest |g - o| / (atol + rtol |o|) over one stream's output: <= 1 passes."""
    a, r = ELEM[kind]
    o = np.asarray(o, dtype=np.float64)
    bound = a * max(float(np.max(np.abs(o))), 1e-30) + r * np.abs(o)
    return float(np.max(np.abs(g.astype(np.float64) - o) / bound))


def oracle_dense(wl, b, emit_round=None, return_layers=False):
    return oracle.dense(wl["layers"], wl["x"][b], wl["weights"], wl["biases"],
                        integer=wl["precision"] == "i8", emit_round=emit_round, return_layers=return_layers)


def oracle_stream(wl, b, seg_rows=None, emit_round=None):
    return oracle.stream_run(wl["layers"], wl["x"][b], wl["weights"], wl["biases"],
                             seg_rows=seg_rows or wl["seg_rows"], integer=wl["precision"] == "i8",
                             emit_round=emit_round)


def oracle_many(fn, wl, streams, threads=None, **kw):
    threads = threads or max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda b: fn(wl, b, **kw), streams))


def gpu_run(wl, seg_rows=None, device="cuda:0", return_streams=False, count_issued=False, events_per_kstep=None):
    """Whole sample of every stream through the GPU library, seg_rows rows per push."""
    import torch
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor
    seg = seg_rows or wl["seg_rows"]
    net = idf.net_from_workload(wl)
    st = idf.Streams(net, wl["streams"], max_seg_rows=seg, device=device)
    x = input_tensor(wl, device)
    H = wl["in_h"]
    if count_issued:
        st.count_issued_macs(True)
    if events_per_kstep is not None:
        st.set_event_path(events_per_kstep)
    for r in range(0, H, seg):
        st.push_segment(x[:, r:r + seg].contiguous())
    out, first, cnt = st.read_outputs(max_rows=int(st.sizes.out_h))
    torch.cuda.synchronize()
    assert (first == 0).all() and (cnt == st.sizes.out_h).all()
    res = out.cpu().numpy()
    if return_streams:
        return res, st, net
    st.close()
    net.destroy()
    return res


def check_stream(wl, g, b, exact_stats=None):
    """Compare GPU output g [H_o][W_o][C_o] of stream b against the oracle."""
    prec = wl["precision"]
    if prec == "i8":
        d = oracle_dense(wl, b)
        assert g.dtype == np.int32
        assert np.array_equal(g.astype(np.int64), d), f"stream {b}: int mismatch"
        assert d.max() > 0
    elif prec == "f32":
        d = oracle_dense(wl, b)
        e = rel_err(g, d)
        assert e <= TOL["f32"], f"stream {b}: rel err {e}"
        assert np.abs(d).max() > 0
    else:
        d_emul = oracle_dense(wl, b, emit_round="bf16")
        d_true = oracle_dense(wl, b)
        e1, e2 = rel_err(g, d_emul), rel_err(g, d_true)
        assert e1 <= TOL["bf16_emul"], f"stream {b}: rel err vs bf16-emitting oracle {e1}"
        assert e2 <= TOL["bf16_true"], f"stream {b}: rel err vs exact oracle {e2}"
