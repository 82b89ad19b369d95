// Launchers of the device kernels (defined in the k_*.hip files), called by the host side.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include "idf_common.h"

namespace idf {

// Where and how a kernel is launched: plain, or bracketed by an event pair stamped at the
// kernel's own start and end (profiling).
struct LaunchCtx {
    hipStream_t st = nullptr;
    hipEvent_t start = nullptr, stop = nullptr;
};

template <class K, class... A>
inline hipError_t launch(K kernel, dim3 grid, dim3 block, size_t lds, const LaunchCtx &c, A... args)
{
    if (c.start) hipExtLaunchKernelGGL(kernel, grid, block, lds, c.st, c.start, c.stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, lds, c.st, args...);
    return hipGetLastError();
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits until every global
// store and atomic of the wave has been acknowledged (a release fence over all address spaces),
// a memory round trip that the kernels here do not need at their internal barriers: what the
// waves of a workgroup exchange goes through LDS.
__device__ __forceinline__ void lds_barrier()
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier\n\ts_waitcnt lgkmcnt(0)" ::: "memory");
#endif
}

enum KernelKind { kKindConvGeneric = 0, kKindPoolGeneric, kKindCopyOut, kKindCascade1d, kKindConvMfma, kKindHead, kKindEager, kKindCount };
inline const char *kind_name(int k)
{
    static const char *names[kKindCount] = {"conv_generic", "pool_generic", "copy_out", "cascade1d", "conv3x3_mfma", "head_accumulate", "eager"};
    return k >= 0 && k < kKindCount ? names[k] : "?";
}

// Generic kernels: any layer shape, any precision (prec = IDF_PREC_*).
hipError_t launch_conv_generic(int prec, const ConvStep &a, const StreamSel &sel, const LaunchCtx &lc);
hipError_t launch_pool_generic(int prec, const PoolStep &a, const StreamSel &sel, const LaunchCtx &lc);
hipError_t launch_head_units(const HeadUnits &a, const StreamSel &sel, int64_t first_slot, int n_rows, const LaunchCtx &lc);
hipError_t launch_head_accumulate(const HeadAcc &a, const StreamSel &sel, int64_t first_slot, int n_rows, const LaunchCtx &lc);
// what: 0 = pushed rows become the announced input, 1 = conv layer, 2 = pool layer
hipError_t launch_eager(int prec, int what, const EagerStep &a, const StreamSel &sel, const LaunchCtx &lc);
// Clears bytes (a multiple of 4, 4-byte aligned) with a kernel on stream st.
hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st);
hipError_t launch_copy_out(const CopyOut &a, const StreamSel &sel, int64_t first_slot, int n_rows,
                           const LaunchCtx &lc);

// Whole-net cascade for 1-D float32 nets: can it serve this net (rows_cap[l] = most rows layer
// l emits per push)?
bool cascade1d_eligible(int prec, const Geom *g, int n_layers, const int *rows_cap, int max_seg_rows);
size_t cascade1d_weight_index(int c_in, int c_out, int ci, int co, int ky);
int cascade1d_slot_off(int S, int rho);   // accumulator slot 0 relative to floor((y0 + p) / S)
hipError_t launch_cascade1d(const CascadeArgs &a, const StreamSel &sel, const LaunchCtx &lc);

// Matrix-core kernel for 3x3 / stride 1 / same-padded conv layers (bf16 and int8 nets).
int conv3x3_mfma_vl(int prec);
bool conv3x3_mfma_eligible(int prec, const Geom &g);
int conv3x3_mfma_tile(const Geom &g, int n_streams);
// Packs weights [k_h][k_w][c_in][c_out] into fragment order; returns the size (out may be null).
size_t conv3x3_mfma_pack(int prec, const Geom &g, const void *w_khkwcico, void *out);
// Where in that packing the event-path weights of an int8 layer begin (0: the layer has none), and the
// most events (tile and halo) the event path takes.
size_t conv3x3_mfma_event_weights(int prec, const Geom &g);
int conv3x3_mfma_event_cap();
// Tiles of one stream's row of w positions x c_out channels in a launch of that tile shape, and how many
// workgroups of such a launch one compute unit holds at once (by the registers the kernel is built for).
int conv3x3_mfma_tiles(int tile, int w, int c_out);
int conv3x3_mfma_batch_resident(int prec, int tile);
hipError_t launch_conv3x3_mfma(int prec, const MfmaStep &a, const StreamSel &sel, const LaunchCtx &lc);
hipError_t launch_conv3x3_mfma_batch(int prec, const MfmaBatch &b, const StreamSel &sel, const LaunchCtx &lc);

// Plain kernels that show what the machine delivers (copy, multiply-add chains, matrix-instruction
// chains): bytes the compute kinds write for a launch of `blocks` workgroups, operations such a
// launch performs, and the launch itself (copy: first half of buf to the second half).
size_t peak_sink_bytes(int blocks);
double peak_ops(int kind, int blocks, int iters);
hipError_t launch_peak(int kind, void *buf, size_t bytes, int blocks, int iters, const LaunchCtx &lc);

// Largest number of touched output rows one generic conv step can take for a layer with
// c_out output channels (the host splits longer steps).
int conv_generic_max_rows(int c_out);
// Chooses tile_x / tile_c / cells_per_thread of a generic conv step.
void conv_generic_plan(ConvStep &a);

}  // namespace idf
