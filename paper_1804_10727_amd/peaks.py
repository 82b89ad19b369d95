"""What the GPU in this machine delivers to plain kernels, next to the published MI355X peaks.

    python -m paper_1804_10727_amd.peaks            # one JSON line

Runs idf_measure_peak for the 16-byte copy (on a 2 GiB buffer: far beyond the last-level cache),
the float32 multiply-add chains and the three matrix-instruction chains.
"""
from __future__ import annotations

import json

PUBLISHED = {  # MI355X, dense
    "copy": (8000.0, "GB/s"),            # HBM3E
    "fma_f32": (157.3, "TFLOP/s"),       # vector float32, counted with packed instructions
    "mfma_f32": (157.3, "TFLOP/s"),
    "mfma_bf16": (2500.0, "TFLOP/s"),
    "mfma_i8": (5000.0, "TOP/s"),
}


def measure(device="cuda:0", copy_bytes=2 << 30):
    import torch
    from .binding import measure_peak
    out = {}
    buf = torch.empty(copy_bytes, dtype=torch.uint8, device=device)
    buf.zero_()
    for kind, (peak, unit) in PUBLISHED.items():
        rate = measure_peak(kind, buf)
        out[kind] = {"measured": rate, "published": peak, "unit": unit, "frac": rate / peak}
    # the same copy on 256 MiB: source and destination together fit the 256 MB last-level cache
    small = min(copy_bytes, 256 << 20)
    rate = measure_peak("copy", buf[:small])
    out["copy_in_last_level_cache"] = {"measured": rate, "published": None, "unit": "GB/s", "frac": None, "bytes": small}
    torch.cuda.synchronize()
    return out


if __name__ == "__main__":
    print(json.dumps(measure()))
