"""Incremental depth-first CNN inference for one AMD MI355X (gfx950).

Thin Python face of the C-ABI library ``libidf.so`` (see include/idf.h): argument
marshalling only -- every step of the method runs in the library's HIP kernels.
PyTorch is used for device memory and streams.
"""
from .binding import (IdfError, Net, Streams, create_net, lib_path, load_library,  # noqa: F401
                      measure_peak, net_from_workload, open_streams)
