"""The five configurations at their full sizes, pushed the way the benchmark pushes them,
checked on sampled streams against the CPU oracle (all streams where the oracle is quick)."""
import numpy as np
import pytest

import workloads as wl_mod
from helpers import TOL, elem_excess, gpu_run, oracle_many, oracle_stream, rel_err

pytestmark = pytest.mark.gpu

# streams compared per configuration: all where the oracle takes seconds, else first, last and
# a few in between
SAMPLED = {1: [0], 2: list(range(64)), 3: list(range(256)), 4: list(range(32)),
           5: [0, 9, 18, 27, 36, 45, 54, 63]}
UNROUNDED = 4       # bfloat16: this many of the sampled streams also against the oracle that rounds nothing


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_full_size(cfg):
    wl = wl_mod.make(cfg)
    print(f"cfg {cfg}: {wl['name']} streams={wl['streams']} seg_rows={wl['seg_rows']}", flush=True)
    out = gpu_run(wl)
    assert out.shape[1:] == wl_mod.output_shape(wl)
    streams = SAMPLED[cfg]
    prec = wl["precision"]
    emul = oracle_many(oracle_stream, wl, streams, emit_round=("bf16" if prec == "bf16" else None))
    for b, (o, _) in zip(streams, emul):
        if prec == "i8":
            assert np.array_equal(out[b].astype(np.int64), o), f"stream {b}"
        else:
            kind = "f32" if prec == "f32" else "bf16_emul"
            e = rel_err(out[b], o)
            assert e <= TOL[kind], f"stream {b}: {e}"
            x = elem_excess(out[b], o, kind)
            assert x <= 1.0, f"stream {b}: element-wise bound exceeded {x} times"
    if prec == "bf16":
        sub = streams[::2][:UNROUNDED - 1] + [streams[-1]]
        true = oracle_many(oracle_stream, wl, sub)
        for b, (o, _) in zip(sub, true):
            e = rel_err(out[b], o)
            assert e <= TOL["bf16_true"], f"stream {b}: {e} against the unrounded oracle"
            x = elem_excess(out[b], o, "bf16_true")
            assert x <= 1.0, f"stream {b}: element-wise bound against the unrounded oracle exceeded {x} times"
    # streams not compared one by one: the cheap invariants that hold at any size
    assert np.isfinite(out.astype(np.float64)).all()
    assert (out >= 0).all()                      # every config ends in a ReLU
    nz = (out.reshape(out.shape[0], -1) != 0).mean(axis=1)
    assert (nz > 0.01).all()
