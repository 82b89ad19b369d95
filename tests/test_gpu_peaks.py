"""idf_measure_peak: the plain kernels run and report rates in a sane range of the published peaks."""
import pytest
import torch

import paper_1804_10727_amd as idf
from paper_1804_10727_amd import peaks
from paper_1804_10727_amd.binding import IdfError

pytestmark = pytest.mark.gpu


def test_rates_are_within_the_published_peaks():
    got = peaks.measure(copy_bytes=1 << 30)
    for kind, r in got.items():
        assert r["measured"] > 0, kind
        if r["published"] is None:
            continue
        # nothing can beat the published peak by more than clock tolerance
        assert r["frac"] < 1.1, (kind, r)
    # plain copy: most of the memory's rate; matrix chains: most of the matrix cores' rate
    assert got["copy"]["frac"] > 0.5, got["copy"]
    for kind in ("mfma_f32", "mfma_bf16", "mfma_i8"):
        assert got[kind]["frac"] > 0.5, (kind, got[kind])
    # the vector units without packed float32 instructions (this build switches them off): up to half the published figure
    assert 0.25 < got["fma_f32"]["frac"] < 0.6, got["fma_f32"]


def test_bad_arguments_are_refused():
    small = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(IdfError):
        idf.measure_peak("copy", small)
    L = idf.load_library()
    big = torch.empty(2 << 20, dtype=torch.uint8, device="cuda:0")
    import ctypes as C
    rate = C.c_double()
    assert L.idf_measure_peak(99, C.c_void_p(big.data_ptr()), big.numel(), None, C.byref(rate)) != 0
    assert L.idf_measure_peak(0, None, big.numel(), None, C.byref(rate)) != 0
