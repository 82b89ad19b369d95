#!/usr/bin/env python3
"""Benchmark of the incremental depth-first CNN update on one MI355X.

One "step" is one whole batch of the workload: every stream's sample is pushed segment by
segment (each segment goes depth-first through every layer it can influence), then the
completed outputs are read.  Inputs are resident in HBM before the timed region starts.

Prints one JSON line: input pixels per second (a pixel = one spatial position of the network
input), with the dense-equivalent and the actually executed multiply-add rates, the roofline
position of the dominant kernel and the CPU oracle timed on the host cores of the same box.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM = 8.0e12
PEAK = {"f32_valu": 157.3e12, "f32_mfma": 157.3e12, "bf16_mfma": 2.5e15, "i8_mfma": 5.0e15, "i32_valu": 157.3e12 / 2}
WORKLOADS = {1: "cfg1_1d_k3_1stream", 2: "cfg2_1d_audio_k9_64streams", 3: "cfg3_2d_small_256streams",
             4: "cfg4_2d_int8_events_32streams", 5: "cfg5_2d_vgg_bf16_64streams"}
DTYPE = {"f32": "f32", "bf16": "bf16", "i8": "int8"}
# kernel family -> (bound kind, peak key per precision)
KERNEL_PEAK = {
    "conv_generic": {"f32": ("alu", "f32_valu"), "bf16": ("alu", "f32_valu"), "i8": ("alu", "i32_valu")},
    "cascade1d": {"f32": ("alu", "f32_valu")},
    "conv3x3_mfma": {"f32": ("mfma", "f32_mfma"), "bf16": ("mfma", "bf16_mfma"), "i8": ("mfma", "i8_mfma")},
    "pool_generic": None, "copy_out": None, "eager": None, "head_accumulate": None,
}


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
KERNEL_SYMBOL = {"cascade1d": "k_cascade1d", "conv3x3_mfma": "k_conv3x3_mfma", "conv_generic": "k_conv_generic"}


def sources_digest():
    """Digest of the kernel and host sources: counter readings are only quoted for the code they were taken on."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_1804_10727_amd", "csrc", "*")) + [os.path.join(ROOT, "include", "idf.h")]):
        h.update(open(f, "rb").read())
    return h.hexdigest()


def stored_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed counter runs, or None (none taken, or
    the sources have changed since)."""
    try:
        rec = json.load(open(TRAFFIC_FILE)).get(workload)
    except (OSError, ValueError):
        return None
    if not rec or rec.get("kernel") != kernel or rec.get("sources_sha256") != sources_digest():
        return None
    return rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"]


def traffic_from_counters(config, fetch_dir, write_dir):
    """Turns two `rocprofv3 --pmc` runs of this bench (FETCH_SIZE, then WRITE_SIZE; KiB per
    dispatch) into HBM bytes per launch of the dominant kernel.  Each counter is scaled by what
    it reads for the plain copy kernel of read_outputs, whose size is known."""
    import csv
    import glob
    import workloads
    wl = workloads.make(config)
    shape = workloads.output_shape(wl)
    copy_kib = wl["streams"] * float(shape[0] * shape[1] * shape[2]) * 4 / 1024.0       # read = written

    def averages(d, counter):
        tot, cnt = {}, {}
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                if row["Counter_Name"] != counter:
                    continue
                k = row["Kernel_Name"]
                tot[k] = tot.get(k, 0.0) + float(row["Counter_Value"]); cnt[k] = cnt.get(k, 0) + 1
        return {k: (tot[k] / cnt[k], cnt[k]) for k in tot}

    out = {}
    for counter, d in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        av = averages(d, counter)
        copy = [v for k, v in av.items() if "k_copy_out" in k]
        assert copy, f"no k_copy_out dispatch in {d}"
        factor = copy_kib / copy[0][0]
        dom = {k: v for k, v in av.items() if any(sym in k for sym in KERNEL_SYMBOL.values())}
        name = max(dom, key=lambda k: dom[k][0] * dom[k][1])
        out[counter] = (factor, dom[name][0] * factor * 1024.0, name, dom[name][1])
    family = [f for f, sym in KERNEL_SYMBOL.items() if sym in out["FETCH_SIZE"][2]][0]
    rec = {"kernel": family, "fetch_factor": out["FETCH_SIZE"][0], "write_factor": out["WRITE_SIZE"][0],
           "fetch_bytes_per_launch": out["FETCH_SIZE"][1], "write_bytes_per_launch": out["WRITE_SIZE"][1],
           "dispatches": out["FETCH_SIZE"][3], "sources_sha256": sources_digest()}
    try:
        allrec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        allrec = {}
    allrec[WORKLOADS[config]] = rec
    json.dump(allrec, open(TRAFFIC_FILE, "w"), indent=1, sort_keys=True)
    print(json.dumps({WORKLOADS[config]: rec}, indent=1))


def trace_summary(stats_csv, bench_log):
    """Text summary of a `rocprofv3 --kernel-trace --stats` run of this bench: the kernel table of
    the trace and the roofline position of the dominant kernel worked out from the TRACE's average
    duration of that kernel (the bench's own line, printed in the same run, supplies the
    algorithmic bytes and executed flops per launch)."""
    import csv
    rows = list(csv.DictReader(open(stats_csv)))
    bench = None
    for l in open(bench_log):
        if l.startswith("{"):
            bench = json.loads(l)
    assert bench, f"no bench line in {bench_log}"
    rf = bench["roofline"]
    eager = bench["config"]["workload"].endswith("_eager_emission")
    cfg_no = {v: k for k, v in WORKLOADS.items()}[bench["config"]["workload"].replace("_eager_emission", "")]
    out = [f"rocprofv3 kernel-trace summary: bench.py workload {bench['config']['workload']} on one MI355X (gfx950)", "",
           "Commands (the first run from /tmp with TMPDIR=/tmp on the GPU machine, the second anywhere; $R = repository root, $OUT = a scratch directory):",
           (f"  rocprofv3 --kernel-trace --stats -d $OUT/prof_eager{cfg_no} -o eager{cfg_no} --output-format csv -- python3 $R/bench.py --config {cfg_no} --eager --no-cpu-baseline > $OUT/prof_eager{cfg_no}.log"
            if eager else
            f"  rocprofv3 --kernel-trace --stats -d $OUT/prof_cfg{cfg_no} -o cfg{cfg_no} --output-format csv -- python3 $R/bench.py --config {cfg_no} --no-cpu-baseline --no-others > $OUT/prof_cfg{cfg_no}.log"),
           (f"  python3 $R/bench.py --config {cfg_no} --trace-summary $OUT/prof_eager{cfg_no}/eager{cfg_no}_kernel_stats.csv $OUT/prof_eager{cfg_no}.log"
            if eager else
            f"  python3 $R/bench.py --config {cfg_no} --trace-summary $OUT/prof_cfg{cfg_no}/cfg{cfg_no}_kernel_stats.csv $OUT/prof_cfg{cfg_no}.log"), "",
           f"bench.py in that run: steps={bench['steps']} warmup={bench['warmup']} (+1 step bracketed by HIP events per launch, "
           f"+1 step on the kernel variants that count issued multiply-adds, named <..., true>); ms_per_step={bench['ms_per_step']:.3f}", "",
           "Kernel statistics (kernel_stats.csv), all launches of the process:",
           f"  {'kernel':<52} {'calls':>7} {'total ms':>10} {'avg us':>9} {'min us':>8} {'max us':>8} {'%':>6}"]
    sym = KERNEL_SYMBOL.get(rf["kernel"], rf["kernel"])
    dom = None
    for r in rows:
        name = r["Name"]
        short = name.replace("(anonymous namespace)::", "").replace("void ", "", 1).split("(")[0].replace("idf::", "")
        short = short if len(short) <= 52 else short[:49] + "..."
        out.append(f"  {short:<52} {int(r['Calls']):>7} {int(r['TotalDurationNs']) / 1e6:>10.3f} {float(r['AverageNs']) / 1e3:>9.2f} "
                   f"{int(r['MinNs']) / 1e3:>8.2f} {int(r['MaxNs']) / 1e3:>8.2f} {float(r['Percentage']):>6.2f}")
        if sym in name and "true>" not in short and (dom is None or int(r["TotalDurationNs"]) > int(dom["TotalDurationNs"])):
            dom = r
    assert dom, f"no {sym} kernel in the trace"
    avg_s = float(dom["AverageNs"]) * 1e-9
    if rf["bound"] == "hbm":
        ach = rf["algorithmic_bytes_per_launch"] / avg_s / 1e9
    else:
        ach = rf["executed_flops_per_launch"] / avg_s / 1e12
    out += ["", f"Dominant kernel: {sym}, trace average {avg_s * 1e6:.2f} us over {dom['Calls']} launches "
                f"(the bench's own HIP-event brackets in an unprofiled run: see the committed bench line; under the profiler the "
                f"brackets themselves are slower, the trace is not).",
            f"Algorithmic bytes per launch {rf['algorithmic_bytes_per_launch']:.0f}; executed flops per launch "
            f"{rf['executed_flops_per_launch']:.0f}; roofline bound '{rf['bound']}' from the trace average: achieved {ach:.1f} {rf['unit']} "
            f"of {rf['peak']:.0f} (frac {ach / rf['peak']:.4f}).",
            f"launches_per_step {rf['launches_per_step']} x trace average = {rf['launches_per_step'] * avg_s * 1e3:.3f} ms against "
            f"ms_per_step {bench['ms_per_step']:.3f} of this profiled run (launches back to back can run shorter than the average of all, spaced ones "
            f"included; where the host's enqueue is what a batch waits for, the profiler's own cost per launch makes the profiled run's ms_per_step larger "
            f"than the unprofiled bench line's)."]
    print("\n".join(out))


def utilisation_from_counters(dirs):
    """Averages per dispatch, for the library's main kernels, of whatever `rocprofv3 --pmc` runs of
    this bench collected -- basic counters or the profiler's derived ones (MfmaUtil, VALUBusy,
    LdsUtil: percent of the time the GPU was active during the dispatch; LdsBankConflict:
    conflict cycles per LDS access cycle)."""
    import csv
    import glob
    tot, cnt = {}, {}
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                k = row["Kernel_Name"]
                if not any(sym in k for sym in KERNEL_SYMBOL.values()) or "true>" in k.replace("(anonymous namespace)::", ""):
                    continue
                key = (k.replace("(anonymous namespace)::", "").replace("void ", "", 1).split("(")[0].replace("idf::", ""), row["Counter_Name"])
                tot[key] = tot.get(key, 0.0) + float(row["Counter_Value"]); cnt[key] = cnt.get(key, 0) + 1
    kernels = sorted({k for k, _ in tot}, key=lambda k: -max(cnt[(k, c)] for kk, c in tot if kk == k))
    for k in kernels:
        av = {c: tot[(kk, c)] / cnt[(kk, c)] for kk, c in tot if kk == k}
        n = max(cnt[(kk, c)] for kk, c in tot if kk == k)
        print(f"{k}: {n} dispatches, averages per dispatch")
        for c in sorted(av):
            print(f"    {c:<34} {av[c]:>16.1f}")


def cpu_baseline(wl, budget_s=12.0):
    """The CPU oracle's event-by-event streaming scheme, as it stands, on this machine's cores."""
    import oracle
    from concurrent.futures import ThreadPoolExecutor
    integer = wl["precision"] == "i8"
    emit = "bf16" if wl["precision"] == "bf16" else None

    def one(b):
        oracle.stream_run(wl["layers"], wl["x"][b], wl["weights"], wl["biases"], seg_rows=wl["seg_rows"],
                          integer=integer, emit_round=emit)
    oracle.lib()
    t0 = time.perf_counter(); one(0); t1 = time.perf_counter() - t0
    cores = max(1, min(16, os.cpu_count() or 1))
    n = int(max(1, min(wl["streams"], (budget_s / max(t1, 1e-6)) * cores * 0.7)))
    threads = min(cores, n)
    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(one, range(n)))
    dt = time.perf_counter() - t0
    px = n * wl["in_h"] * wl["in_w"]
    return {"value": px / dt, "unit": "pixels/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} of {wl['streams']} streams, whole samples, seg_rows={wl['seg_rows']}, "
                      f"scalar event-by-event fp64/int64, one stream per thread, {dt:.1f} s"}


def run_workload(config, steps_arg=None, warmup_arg=None, eager=False, push_batch=1, event_path=0, rows_per_push=None):
    """Times `steps` whole batches of one workload; returns (result dict, workload)."""
    import numpy as np
    import torch
    import workloads
    import paper_1804_10727_amd as idf
    from paper_1804_10727_amd.binding import input_tensor, load_library
    import ctypes as C

    dev = "cuda:0"
    wl = workloads.make(config)
    B, H, W, C0, seg = wl["streams"], wl["in_h"], wl["in_w"], wl["in_c"], wl["seg_rows"]
    if rows_per_push:           # 2-D workloads with more rows per push than the configuration states (throughput mode)
        seg = rows_per_push
    n_seg = (H + seg - 1) // seg
    assert H % seg == 0
    steps = steps_arg if steps_arg is not None else {1: 5, 2: 10, 3: 50, 4: 10, 5: 5}[config]
    warmup = warmup_arg if warmup_arg is not None else 2

    net = idf.net_from_workload(wl)
    st = idf.Streams(net, B, max_seg_rows=seg, device=dev)
    if eager:
        st.enable_eager()
    if push_batch > 1:          # throughput mode of the 1-D cascade: several pushes in step share a launch
        st.set_push_batching(push_batch)
    if event_path > 0:          # int8: sparse tiles visit a packed event list on the vector units instead of contracting
        st.set_event_path(event_path)
    x = input_tensor(wl, dev)
    # segment-major copy in HBM: xs[i] is the contiguous block [B][seg][W][C] of push i
    xs = x.view(B, n_seg, seg, W, C0).permute(1, 0, 2, 3, 4).contiguous()
    del x
    out_h = int(st.sizes.out_h)
    out = torch.empty((B, out_h, st.sizes.out_w, st.sizes.out_c), dtype=st.out_dtype, device=dev)
    L = load_library()
    h = st._h
    seg_ptrs = [C.c_void_p(xs[i].data_ptr()) for i in range(n_seg)]
    first = np.zeros(B, dtype=np.int64); cnt = np.zeros(B, dtype=np.int32)
    out_ptr = C.c_void_p(out.data_ptr())
    push = L.idf_push_segment
    read = L.idf_read_outputs

    def step():
        for p in seg_ptrs:
            rc = push(h, None, B, p, seg)
            if rc:
                raise RuntimeError(L.idf_last_error().decode())
        if eager:       # the announced map of the last layer, valid after every segment, read once per batch
            rc = L.idf_read_announced(h, len(wl["layers"]), None, B, out_ptr)
        else:
            rc = read(h, None, B, out_ptr, out_h, first.ctypes.data, cnt.ctypes.data)
        if rc:
            raise RuntimeError(L.idf_last_error().decode())

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    t_enq = time.perf_counter() - t0            # host side only: all launches handed to the runtime
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / steps * 1e3
    pixels = B * H * W
    value = pixels / (dt / steps)

    # executed work and kernel times of one more step, bracketed kernel by kernel
    def macs_total():
        ev = np.zeros(len(wl["layers"]), dtype=np.float64); mc = np.zeros(len(wl["layers"]), dtype=np.float64)
        for b in range(B):
            s = st.get_stats(b)
            ev += s["events_in"]; mc += s["macs"]
        return ev, mc

    def issued_total():
        if eager:
            return None
        tot = np.zeros(len(wl["layers"]), dtype=np.float64)
        for b in range(B):
            tot += st.get_issued_macs(b).astype(np.float64)
        return tot
    ev0, mc0 = macs_total()
    st.profile_begin()
    step()
    by_layer = st.profile_end()
    prof = {}
    for p in by_layer:                       # "family@layer" -> family
        f = prof.setdefault(p["name"].split("@")[0], dict(name=p["name"].split("@")[0], launches=0, total_ms=0.0,
                                                          algorithmic_bytes=0.0))
        f["launches"] += p["launches"]; f["total_ms"] += p["total_ms"]; f["algorithmic_bytes"] += p["algorithmic_bytes"]
    prof = list(prof.values())
    ev1, mc1 = macs_total()
    macs_issued = None
    if not eager:
        # one more step on the kernel variants that add up what they issue (an atomic per wave):
        # neither the timed steps nor the bracketed one above run those
        st.count_issued_macs(True)
        is0 = issued_total()
        step()
        issued_layer = issued_total() - is0    # zeros inside visited fragments / channels included
        macs_issued = float(issued_layer.sum())
        st.count_issued_macs(False)
    macs_exec_layer = mc1 - mc0
    macs_exec = float(macs_exec_layer.sum())
    macs_dense = float(workloads.dense_equivalent_macs(wl)) * B
    kinds = st.layer_kernels()

    dom = max(prof, key=lambda p: p["total_ms"])
    avg_s = dom["total_ms"] * 1e-3 / dom["launches"]
    bytes_per_launch = dom["algorithmic_bytes"] / dom["launches"]
    layer_idx = [i for i, k in enumerate(kinds) if k == dom["name"] or dom["name"].startswith(k)]
    flops_per_launch = 2.0 * float(sum(macs_exec_layer[i] for i in layer_idx)) / dom["launches"]
    pk = KERNEL_PEAK.get(dom["name"])
    kind_peak = pk[wl["precision"]] if pk else None
    t_hbm = bytes_per_launch / PEAK_HBM
    t_alu = flops_per_launch / PEAK[kind_peak[1]] if kind_peak else 0.0
    if kind_peak and t_alu > t_hbm:
        roof = {"bound": kind_peak[0], "achieved": flops_per_launch / avg_s / 1e12, "peak": PEAK[kind_peak[1]] / 1e12,
                "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": bytes_per_launch / avg_s / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # (the counters were taken in the configuration's own mode: one push per launch, its rows per push)
    roof["traffic"] = stored_traffic(WORKLOADS[config], dom["name"]) if push_batch == 1 and not rows_per_push and not eager else None
    roof.update({"kernel": dom["name"], "avg_launch_us": avg_s * 1e6, "launches_per_step": dom["launches"],
                 "algorithmic_bytes_per_launch": bytes_per_launch, "executed_flops_per_launch": flops_per_launch,
                 "kernel_time_share": dom["total_ms"] / sum(p["total_ms"] for p in prof),
                 "gpu_busy_ms_per_step": sum(p["total_ms"] for p in prof)})

    res = {
        "metric": "input_pixels_per_s", "value": value, "unit": "pixels/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "host_enqueue_ms_per_step": t_enq / steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": DTYPE[wl["precision"]], "data": "synthetic",
        "config": {"workload": WORKLOADS[config] + ("_eager_emission" if eager else ""), "streams": B, "rows_per_sample": H, "row_width": W,
                   "in_channels": C0, "rows_per_push": seg, "pushes_per_step": n_seg, "pushes_per_launch": push_batch, "event_list_events_per_kstep": event_path,
                   "layers": len(wl["layers"]),
                   # rolling buffers + held rows (what the paper bounds), the rows waiting between layers
                   # across calls in the staged mode that was timed, and their sum
                   "state": {"state_bytes_per_stream": int(st.sizes.state_bytes_per_stream),
                             "handover_bytes_per_stream": int(st.sizes.handover_bytes_per_stream),
                             "retained_bytes_per_stream": int(st.sizes.retained_bytes_per_stream),
                             "mode": "staged" if st.sizes.handover_bytes_per_stream else "strict depth-first"}},
        "gmacs_dense_equivalent": macs_dense / (dt / steps) / 1e9,
        "gmacs_executed": macs_exec / (dt / steps) / 1e9,
        "gmacs_issued": None if macs_issued is None else macs_issued / (dt / steps) / 1e9,
        "executed_over_dense": macs_exec / macs_dense,
        "issued_over_dense": None if macs_issued is None else macs_issued / macs_dense,
        # conv layers in order: what each issues and executes, as fractions of its own dense-equivalent multiply-adds
        "issued_over_dense_by_layer": None if macs_issued is None else
        [round(float(i) / (d * B), 4) for i, d in zip(issued_layer, workloads.dense_equivalent_macs_by_layer(wl)) if d],
        "executed_over_dense_by_layer": [round(float(e) / (d * B), 4) for e, d in zip(macs_exec_layer, workloads.dense_equivalent_macs_by_layer(wl)) if d],
        "kernels": {p["name"]: {"launches": p["launches"], "total_ms": p["total_ms"]} for p in prof},
        "kernels_by_layer": {p["name"]: {"launches": p["launches"], "avg_us": p["total_ms"] * 1e3 / p["launches"],
                                         "alg_GBps": p["algorithmic_bytes"] / (p["total_ms"] * 1e-3) / 1e9}
                             for p in by_layer},
        "roofline": roof,
    }
    if eager:
        # what eager emission costs against emission once per finished row: the state it keeps and
        # the events it delivers (every change of a value is an event, not only its final value)
        nb, kept = st.eager_state_bytes()
        st.close()
        st2 = idf.Streams(net, B, max_seg_rows=seg, device=dev)
        for i in range(n_seg):
            st2.push_segment(xs[i])
        st2.read_outputs(out_h, out=out)
        ev_rc = sum(st2.get_stats(b)["events_in"].astype(np.float64) for b in range(B))
        res["eager"] = {"state_bytes_per_stream": int(nb), "rows_kept_per_level": [int(k) for k in kept],
                        "row_complete_state_bytes_per_stream": int(st2.sizes.state_bytes_per_stream),
                        "events_delivered_per_layer": [float(v) for v in (ev1 - ev0)],
                        "row_complete_events_per_layer": [float(v) for v in ev_rc],
                        "events_over_row_complete": float((ev1 - ev0).sum() / max(ev_rc.sum(), 1.0))}
        st2.close()
        net.destroy()
        return res, wl
    st.close()
    net.destroy()
    return res, wl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=5,
                    help="workload 1..5 (default 5: the largest configuration, 64 streams of 224x224x3 bfloat16)")
    ap.add_argument("--eager", action="store_true", help="eager emission (configs 3 and 4): output valid after every push")
    ap.add_argument("--push-batch", type=int, default=1,
                    help="1-D workloads: hold back up to this many pushes in step per launch (throughput mode; 1 = a launch per push)")
    ap.add_argument("--rows-per-push", type=int, default=None,
                    help="2-D workloads: push this many rows per call instead of the configuration's one (throughput mode: "
                         "nets served by the matrix-core kernel then go through the layers two rows per launch)")
    ap.add_argument("--event-path", type=int, default=0,
                    help="int8 workloads: tiles with at most this many events per K-step take the event-list path (0 = off, the library's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", dest="others", action="store_false",
                    help="skip the short runs of the other workloads (reported under other_workloads)")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU run: read two rocprofv3 --pmc outputs of this bench (FETCH_SIZE, WRITE_SIZE) "
                         "and store the dominant kernel's HBM bytes per launch in profiles/traffic.json")
    ap.add_argument("--trace-summary", nargs=2, metavar=("KERNEL_STATS_CSV", "BENCH_LOG"),
                    help="no GPU run: text summary of a rocprofv3 --kernel-trace --stats run of this bench "
                         "(its kernel_stats.csv and the output of the bench in that run)")
    ap.add_argument("--util-from", nargs="+", metavar="DIR",
                    help="no GPU run: averages of rocprofv3 --pmc counter runs of this bench for the dominant kernels")
    args = ap.parse_args()
    if args.traffic_from:
        traffic_from_counters(args.config, *args.traffic_from)
        return
    if args.trace_summary:
        trace_summary(*args.trace_summary)
        return
    if args.util_from:
        utilisation_from_counters(args.util_from)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (streams are independent: more GPUs "
              "would each take a share of the streams, no figure for that is produced here)", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    res, wl = run_workload(args.config, args.steps, args.warmup, eager=args.eager, push_batch=args.push_batch, event_path=args.event_path,
                           rows_per_push=args.rows_per_push)
    if args.eager:
        print(json.dumps(res))
        return
    if args.others:
        # the other multi-stream workloads, a few steps each, as context in the same line
        res["other_workloads"] = {}
        for c in (1, 2, 3, 4, 5):
            if c == args.config:
                continue
            o, owl = run_workload(c, None, 1)
            rec = {k: o[k] for k in ("value", "unit", "ms_per_step", "steps", "dtype", "gmacs_dense_equivalent",
                                     "gmacs_executed", "gmacs_issued", "issued_over_dense", "executed_over_dense", "issued_over_dense_by_layer", "executed_over_dense_by_layer",
                                     "roofline")}
            rec["state"] = o["config"]["state"]
            if c in (1, 2):     # the 1-D workloads also in throughput mode: up to 16 pushes in step per launch
                t, _ = run_workload(c, None, 1, push_batch=16)
                rec["throughput_mode_16_pushes_per_launch"] = {k: t[k] for k in ("value", "unit", "ms_per_step", "roofline")}
            else:               # the 2-D workloads also with two rows per push: one launch per two rows
                t, _ = run_workload(c, None, 1, rows_per_push=2)
                rec["throughput_mode_2_rows_per_push"] = {k: t[k] for k in ("value", "unit", "ms_per_step", "roofline")}
            if not args.no_cpu_baseline:
                rec["cpu_baseline"] = cpu_baseline(owl, budget_s=3.0)
            res["other_workloads"][o["config"]["workload"]] = rec
    if args.others and args.config in (3, 4, 5) and not args.rows_per_push:
        # the same workload pushed two rows per call (not the configuration's one): context, never `value`
        t, _ = run_workload(args.config, None, 1, rows_per_push=2)
        res["throughput_mode_2_rows_per_push"] = {k: t[k] for k in ("value", "unit", "ms_per_step", "roofline")}
    if args.others:
        # what this GPU gives plain copy / multiply-add / matrix-instruction kernels, next to the published
        # peaks the rooflines are priced against (idf_measure_peak; about a second)
        from paper_1804_10727_amd import peaks
        res["machine"] = {k: {kk: (round(vv, 4) if isinstance(vv, float) else vv) for kk, vv in v.items()} for k, v in peaks.measure().items()}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
