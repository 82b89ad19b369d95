// Launchers of the device kernels (defined in the k_*.hip files), called by the host side.
#pragma once

#include <hip/hip_runtime.h>

#include "idf_common.h"

namespace idf {

// Generic kernels: any layer shape, any precision (prec = IDF_PREC_*).
hipError_t launch_conv_generic(int prec, const ConvStep &a, const StreamSel &sel, hipStream_t st);
hipError_t launch_pool_generic(int prec, const PoolStep &a, const StreamSel &sel, hipStream_t st);
hipError_t launch_copy_out(const CopyOut &a, const StreamSel &sel, int64_t first_slot, int n_rows,
                           hipStream_t st);

// Largest number of touched output rows one generic conv step can take for a layer with
// c_out output channels (the host splits longer steps).
int conv_generic_max_rows(int c_out);
// Chooses tile_x / tile_c / cells_per_thread of a generic conv step.
void conv_generic_plan(ConvStep &a);

}  // namespace idf
