// Generic event-propagation kernels: any layer shape, any precision.  They are the fallback
// for shapes the specialised kernels do not cover and the simplest statement of the update:
//
//   Every workgroup owns a band of cells (x_out, c_out) of one stream's layer, across all the
//   output rows the arriving input rows touch.  Each cell starts from its retained
//   pre-activation c (or from the bias when this step is the first to touch its row), adds
//   w * dh for every non-zero dh in its kernel footprint among the new rows (Sec. 3, the
//   event-delivery rule; zero values are skipped, Sec. 1), and then either goes back to the
//   ring or -- when no future row can reach it -- is activated and emitted (Sec. 3, stateful
//   neuron and event definition; Fig. 2: a finished region is dropped).
//
// Ownership instead of scatter: two events never race for one cell, so float results are
// reproducible run to run.
#include "idf.h"
#include "idf_kernels.h"

namespace idf {

// ---------------------------------------------------------------------------------------
// Per-precision value handling
// ---------------------------------------------------------------------------------------
template <int PREC> struct Prec;

template <> struct Prec<IDF_PREC_F32> {
    using ev_t = float; using w_t = float; using st_t = float; using out_t = float;
    static __device__ __forceinline__ bool nz(ev_t v) { return v != 0.0f; }
    static __device__ __forceinline__ st_t val(ev_t v) { return v; }
    static __device__ __forceinline__ st_t wval(w_t v) { return v; }
    static __device__ __forceinline__ st_t mac(st_t acc, st_t v, st_t w) { return fmaf(v, w, acc); }
    static __device__ __forceinline__ ev_t to_ev(st_t h) { return h; }
    static __device__ __forceinline__ out_t ev_to_out(ev_t v) { return v; }
};

template <> struct Prec<IDF_PREC_BF16> {
    using ev_t = uint16_t; using w_t = uint16_t; using st_t = float; using out_t = float;
    static __device__ __forceinline__ bool nz(ev_t v) { return (v & 0x7fffu) != 0; }
    static __device__ __forceinline__ st_t val(ev_t v) { return __uint_as_float((uint32_t)v << 16); }
    static __device__ __forceinline__ st_t wval(w_t v) { return __uint_as_float((uint32_t)v << 16); }
    static __device__ __forceinline__ st_t mac(st_t acc, st_t v, st_t w) { return fmaf(v, w, acc); }
    // round to nearest, ties to even, on the upper 16 bits of the binary32 pattern
    static __device__ __forceinline__ ev_t to_ev(st_t h)
    {
        uint32_t u = __float_as_uint(h);
        u += 0x7fffu + ((u >> 16) & 1u);
        return (ev_t)(u >> 16);
    }
    static __device__ __forceinline__ out_t ev_to_out(ev_t v) { return val(v); }
};

template <> struct Prec<IDF_PREC_I8> {
    using ev_t = int8_t; using w_t = int8_t; using st_t = int32_t; using out_t = int32_t;
    static __device__ __forceinline__ bool nz(ev_t v) { return v != 0; }
    static __device__ __forceinline__ st_t val(ev_t v) { return v; }
    static __device__ __forceinline__ st_t wval(w_t v) { return v; }
    static __device__ __forceinline__ st_t mac(st_t acc, st_t v, st_t w) { return acc + v * w; }
    static __device__ __forceinline__ ev_t to_ev(st_t h) { return (ev_t)h; }
    static __device__ __forceinline__ out_t ev_to_out(ev_t v) { return v; }
};

__device__ __forceinline__ float activate(const Geom &g, float c)
{
    return g.act == IDF_ACT_NONE ? c : fmaxf(c, 0.0f);
}

__device__ __forceinline__ int32_t activate(const Geom &g, int32_t c)
{
    if (g.act == IDF_ACT_NONE) return c;
    int32_t r = c > 0 ? c : 0;
    if (g.act == IDF_ACT_RELU_SHR_CLAMP) {
        r >>= g.shr;
        r = r > g.clamp_hi ? g.clamp_hi : r;
    }
    return r;
}

// Taps of a conv layer that an input row y / column x lands on inside the output.
__device__ __forceinline__ int taps_1d(int64_t pos, int k, int s, int p, int64_t n_out)
{
    int n = 0;
    for (int kk = 0; kk < k; ++kk) {
        int64_t t = pos + p - kk;
        if (t < 0 || t % s != 0) continue;
        if (n_out > 0 && t / s >= n_out) continue;
        ++n;
    }
    return n;
}

// Adds (events, macs) of one workgroup's threads into the per-stream per-layer counters.
__device__ __forceinline__ void block_add_stats(unsigned long long ev, unsigned long long macs,
                                                unsigned long long *dst)
{
    __shared__ unsigned long long red[2][4];
    for (int off = 32; off > 0; off >>= 1) {
        ev += __shfl_down(ev, off);
        macs += __shfl_down(macs, off);
    }
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) { red[0][wave] = ev; red[1][wave] = macs; }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long e = 0, m = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) { e += red[0][w]; m += red[1][w]; }
        if (e) atomicAdd(dst, e);
        if (m) atomicAdd(dst + 1, m);
    }
}

// ---------------------------------------------------------------------------------------
// Convolution step
// ---------------------------------------------------------------------------------------
constexpr int kGenThreads = 256;
constexpr int kGenCells = 8;                     // cells per thread at most
constexpr int kGenMaxTile = kGenThreads * kGenCells;

template <int PREC>
__global__ void __launch_bounds__(kGenThreads) k_conv_generic(const ConvStep a, const StreamSel sel)
{
    using T = Prec<PREC>;
    using ev_t = typename T::ev_t; using w_t = typename T::w_t;
    using st_t = typename T::st_t; using out_t = typename T::out_t;
    const Geom &g = a.g;
    const int si = blockIdx.z;
    const int stream = sel_stream(sel, si);
    const int64_t in_idx = a.in_by_position ? (int64_t)(sel.pos0 + si) : (int64_t)stream;
    const ev_t *in = (const ev_t *)a.in + in_idx * a.in_stream_stride;
    st_t *ring = (st_t *)a.ring + (int64_t)stream * a.ring_stream_stride;
    const w_t *w = (const w_t *)a.w;
    const st_t *bias = (const st_t *)a.bias;
    const int row_in = g.w_in * g.c_in, row_out = g.w_out * g.c_out;

    // a pixel segment holds only columns [px_lo, px_hi) of its one row
    const int px_lo = a.x_hi > 0 ? a.x_lo : 0, px_hi = a.x_hi > 0 ? a.x_hi : g.w_in;
    if (blockIdx.x == 0 && blockIdx.y == 0 && a.stats) {
        unsigned long long ev = 0, macs = 0;
        const ev_t *rows = in + (a.y0 - a.in_row0) * row_in;
        const int row_have = (px_hi - px_lo) * g.c_in;            // == row_in for whole rows
        for (int i = threadIdx.x; i < a.cnt * row_have; i += kGenThreads) {
            if (!T::nz(rows[i])) continue;
            int r = i / row_have, x = px_lo + (i % row_have) / g.c_in;
            int ty = taps_1d(a.y0 + r, g.k_h, g.s_h, g.p_h, g.h_out);
            int tx = taps_1d(x, g.k_w, g.s_w, g.p_w, g.w_out);
            ev += 1;
            macs += (unsigned long long)(ty * tx) * g.c_out;
        }
        block_add_stats(ev, macs, a.stats + ((int64_t)stream * a.n_layers + a.layer) * 2);
    }

    const int x_base = blockIdx.x * a.tile_x, c_base = blockIdx.y * a.tile_c;
    const int n_t = (int)(a.o_hi - a.o_lo);
    const int cells = n_t * a.tile_x * a.tile_c;
    // Everything below works in small integers relative to the first touched output row o_lo and
    // the first new input row y0 (64-bit row numbers are only needed to get these offsets).
    const int slot_lo = (int)(a.o_lo % a.ring_rows);          // ring slot of o_lo
    const int d0 = (int)(a.o_lo * g.s_h - g.p_h - a.y0);      // first input row of o_lo, relative to y0
    const bool at_start = a.y0 == 0;
    const int n_fin = (int)(a.o_fin - a.o_lo);
    const int in_off = (int)(a.y0 - a.in_row0);
    const int64_t dst_rel0 = a.o_lo - a.dst_row0;
    const int plane = a.tile_c * a.tile_x;

    st_t acc[kGenCells];
    // Phase 1: every cell fetches its starting value before any cell of the band writes, since
    // a row that is about to be forgotten and a row that is new can share a ring slot.
#pragma unroll
    for (int j = 0; j < kGenCells; ++j) {
        int idx = threadIdx.x + j * kGenThreads;
        acc[j] = 0;
        if (j >= a.cells_per_thread || idx >= cells) continue;
        int oi = idx / plane, rem = idx - oi * plane;
        int xi = rem / a.tile_c;
        int co = c_base + rem - xi * a.tile_c, xo = x_base + xi;
        if (co >= g.c_out || xo >= g.w_out) continue;
        const bool fresh = (d0 + oi * g.s_h >= 0 || at_start) && !a.cont;
        if (fresh) acc[j] = bias ? bias[co] : (st_t)0;
        else acc[j] = ring[((slot_lo + oi) % a.ring_rows) * row_out + xo * g.c_out + co];
    }
    __syncthreads();
    // Phase 2: deliver the events of the new rows, then emit or retain.
#pragma unroll
    for (int j = 0; j < kGenCells; ++j) {
        int idx = threadIdx.x + j * kGenThreads;
        if (j >= a.cells_per_thread || idx >= cells) continue;
        int oi = idx / plane, rem = idx - oi * plane;
        int xi = rem / a.tile_c;
        int co = c_base + rem - xi * a.tile_c, xo = x_base + xi;
        if (co >= g.c_out || xo >= g.w_out) continue;
        st_t c = acc[j];
        for (int ky = 0; ky < g.k_h; ++ky) {
            int yr = d0 + oi * g.s_h + ky;                    // input row relative to y0
            if (yr < 0 || yr >= a.cnt) continue;
            const ev_t *row = in + (int64_t)(yr + in_off) * row_in;
            for (int kx = 0; kx < g.k_w; ++kx) {
                int x = xo * g.s_w - g.p_w + kx;
                if (x < px_lo || x >= px_hi) continue;
                const ev_t *px = row + (x - px_lo) * g.c_in;
                const w_t *wp = w + ((int64_t)(ky * g.k_w + kx) * g.c_in) * g.c_out + co;
                for (int ci = 0; ci < g.c_in; ++ci) {
                    ev_t v = px[ci];
                    if (T::nz(v)) c = T::mac(c, T::val(v), T::wval(wp[ci * g.c_out]));
                }
            }
        }
        if (oi < n_fin) {
            st_t h = activate(g, c);
            if (a.to_output) {
                int64_t slot = a.dst_slot0 + dst_rel0 + oi;
                if (slot >= a.out_cap) slot -= a.out_cap;
                ((out_t *)a.dst)[(int64_t)stream * a.dst_stream_stride + slot * row_out + xo * g.c_out + co] = (out_t)h;
            } else {
                ((ev_t *)a.dst)[(int64_t)stream * a.dst_stream_stride + (dst_rel0 + oi) * row_out + xo * g.c_out + co] = T::to_ev(h);
            }
        } else {
            ring[((slot_lo + oi) % a.ring_rows) * row_out + xo * g.c_out + co] = c;
        }
    }
}

int conv_generic_max_rows(int c_out)
{
    int tile_c = c_out < 64 ? c_out : 64;
    return kGenMaxTile / tile_c;
}

void conv_generic_plan(ConvStep &a)
{
    int n_t = (int)(a.o_hi - a.o_lo);
    if (n_t < 1) n_t = 1;
    a.tile_c = a.g.c_out < 64 ? a.g.c_out : 64;
    int tx = kGenMaxTile / (n_t * a.tile_c);
    if (tx < 1) tx = 1;
    if (tx > a.g.w_out) tx = a.g.w_out;
    // prefer more workgroups over long per-thread loops when the row is wide
    while (tx > 1 && n_t * tx * a.tile_c > 2 * kGenThreads && (a.g.w_out + tx - 1) / tx < 8) tx = (tx + 1) / 2;
    a.tile_x = tx;
    a.cells_per_thread = (n_t * a.tile_x * a.tile_c + kGenThreads - 1) / kGenThreads;
}

hipError_t launch_conv_generic(int prec, const ConvStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    dim3 grid((a.g.w_out + a.tile_x - 1) / a.tile_x, (a.g.c_out + a.tile_c - 1) / a.tile_c, sel.n);
    dim3 block(kGenThreads);
    switch (prec) {
    case IDF_PREC_F32: return launch(k_conv_generic<IDF_PREC_F32>, grid, block, 0, lc, a, sel);
    case IDF_PREC_BF16: return launch(k_conv_generic<IDF_PREC_BF16>, grid, block, 0, lc, a, sel);
    case IDF_PREC_I8: return launch(k_conv_generic<IDF_PREC_I8>, grid, block, 0, lc, a, sel);
    default: return hipErrorInvalidValue;
    }
}

// ---------------------------------------------------------------------------------------
// Max-pool step: rows arrive final, so this is the ordinary maximum over a pair of rows; the
// even row of a pair waits in the held row until the odd one arrives.
// ---------------------------------------------------------------------------------------
template <int PREC>
__global__ void __launch_bounds__(kGenThreads) k_pool_generic(const PoolStep a, const StreamSel sel)
{
    using T = Prec<PREC>;
    using ev_t = typename T::ev_t; using st_t = typename T::st_t; using out_t = typename T::out_t;
    const Geom &g = a.g;
    const int si = blockIdx.z;
    const int stream = sel_stream(sel, si);
    const int64_t in_idx = a.in_by_position ? (int64_t)(sel.pos0 + si) : (int64_t)stream;
    const ev_t *in = (const ev_t *)a.in + in_idx * a.in_stream_stride;
    ev_t *held = (ev_t *)a.held + (int64_t)stream * a.held_stream_stride;
    const int C = g.c_out, row_in = g.w_in * C, row_out = g.w_out * C;

    if (blockIdx.x == 0 && a.stats) {
        unsigned long long ev = 0;
        const ev_t *rows = in + (a.y0 - a.in_row0) * row_in;
        for (int i = threadIdx.x; i < a.cnt * row_in; i += kGenThreads) ev += T::nz(rows[i]) ? 1 : 0;
        block_add_stats(ev, 0, a.stats + ((int64_t)stream * a.n_layers + a.layer) * 2);
    }

    const int n_out = (int)(a.o_fin - a.o_lo);
    const int rows = n_out > 0 ? n_out : 1;
    const int idx = blockIdx.x * kGenThreads + threadIdx.x;
    if (idx >= rows * row_out) return;
    const int c = idx % C, ox = (idx / C) % g.w_out, oi = idx / row_out;
    const int e0 = (int)(2 * a.o_lo - a.y0);       // even row of the first pair, relative to y0 (-1: held)
    const int in_off = (int)(a.y0 - a.in_row0);
    const int64_t dst_rel0 = a.o_lo - a.dst_row0;
    if (oi < n_out) {
        const int y_even = e0 + 2 * oi, y_odd = y_even + 1;
        st_t m = 0;
        for (int kx = 0; kx < g.k_w; ++kx) {
            int x = ox * g.s_w + kx;
            ev_t e = y_even >= 0 ? in[(int64_t)(y_even + in_off) * row_in + x * C + c] : held[x * C + c];
            ev_t d = in[(int64_t)(y_odd + in_off) * row_in + x * C + c];
            st_t ve = T::val(e), vd = T::val(d);
            st_t mm = ve > vd ? ve : vd;
            m = (kx == 0 || mm > m) ? mm : m;
        }
        if (a.to_output) {
            int64_t slot = a.dst_slot0 + dst_rel0 + oi;
            if (slot >= a.out_cap) slot -= a.out_cap;
            ((out_t *)a.dst)[(int64_t)stream * a.dst_stream_stride + slot * row_out + ox * C + c] = (out_t)m;
        } else {
            ((ev_t *)a.dst)[(int64_t)stream * a.dst_stream_stride + (dst_rel0 + oi) * row_out + ox * C + c] = T::to_ev(m);
        }
    }
    // The thread that consumed the old held values of its window is the one that replaces them.
    if (oi == 0 && a.hold_new) {
        for (int kx = 0; kx < g.k_w; ++kx) {
            int x = ox * g.s_w + kx;
            held[x * C + c] = in[(int64_t)(a.cnt - 1 + in_off) * row_in + x * C + c];
        }
    }
}

hipError_t launch_pool_generic(int prec, const PoolStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    int n_out = (int)(a.o_fin - a.o_lo);
    int rows = n_out > 0 ? n_out : 1;
    int total = rows * a.g.w_out * a.g.c_out;
    dim3 grid((total + kGenThreads - 1) / kGenThreads, 1, sel.n);
    dim3 block(kGenThreads);
    switch (prec) {
    case IDF_PREC_F32: return launch(k_pool_generic<IDF_PREC_F32>, grid, block, 0, lc, a, sel);
    case IDF_PREC_BF16: return launch(k_pool_generic<IDF_PREC_BF16>, grid, block, 0, lc, a, sel);
    case IDF_PREC_I8: return launch(k_pool_generic<IDF_PREC_I8>, grid, block, 0, lc, a, sel);
    default: return hipErrorInvalidValue;
    }
}

// ---------------------------------------------------------------------------------------
// Output hand-over: rows [first_slot, first_slot + n_rows) of the output ring -> caller.
// Output elements are always 4 bytes (float32 / int32).
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kGenThreads) k_copy_out(const CopyOut a, const StreamSel sel,
                                                          int64_t first_slot, int n_rows)
{
    const int si = blockIdx.z;
    const int stream = sel_stream(sel, si);
    const uint32_t *src = (const uint32_t *)a.src + (int64_t)stream * a.src_stream_stride;
    uint32_t *dst = (uint32_t *)a.dst + (int64_t)(sel.pos0 + si) * a.dst_stream_stride;
    // The rows lie one after the other in both areas, except where the output ring wraps: at most
    // two contiguous stretches, each copied flat, 16 bytes per lane where sizes and addresses allow
    // it (the same for every lane).
    const bool wide = a.row_elems % 4 == 0 && a.src_stream_stride % 4 == 0 && a.dst_stream_stride % 4 == 0 &&
                      ((uintptr_t)a.src | (uintptr_t)a.dst) % 16 == 0;
    const int64_t rows1 = n_rows < a.out_cap - first_slot ? n_rows : a.out_cap - first_slot;
    const int64_t start = (int64_t)blockIdx.x * kGenThreads + threadIdx.x, step = (int64_t)gridDim.x * kGenThreads;
    for (int part = 0; part < 2; ++part) {
        const int64_t rows = part == 0 ? rows1 : n_rows - rows1;
        if (rows <= 0) continue;
        const uint32_t *sp = src + (part == 0 ? first_slot : 0) * a.row_elems;
        uint32_t *dp = dst + (part == 0 ? 0 : rows1) * a.row_elems;
        const int64_t n = rows * a.row_elems;
        if (wide) {
            const uint4 *s4 = reinterpret_cast<const uint4 *>(sp);
            uint4 *d4 = reinterpret_cast<uint4 *>(dp);
            for (int64_t e = start; e < n / 4; e += step) d4[e] = s4[e];
        } else {
            for (int64_t e = start; e < n; e += step) dp[e] = sp[e];
        }
    }
}

hipError_t launch_copy_out(const CopyOut &a, const StreamSel &sel, int64_t first_slot, int n_rows,
                           const LaunchCtx &lc)
{
    if (first_slot < 0 || first_slot >= a.out_cap || n_rows > a.out_cap) return hipErrorInvalidValue;
    const int64_t units = (int64_t)n_rows * a.row_elems / (a.row_elems % 4 == 0 ? 4 : 1);
    int64_t blocks = (units + kGenThreads - 1) / kGenThreads;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    return launch(k_copy_out, dim3((unsigned)blocks, 1, sel.n), dim3(kGenThreads), 0, lc, a, sel, first_slot, n_rows);
}

// ---------------------------------------------------------------------------------------
// Clears n 4-byte words: what the host side uses wherever state, counters or maps must start at
// zero, so that a caller who records the library's work into a HIP graph records kernels only.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kGenThreads) k_fill_zero(uint32_t *p, int64_t n)
{
    const int64_t start = (int64_t)blockIdx.x * kGenThreads + threadIdx.x, step = (int64_t)gridDim.x * kGenThreads;
    if (((uintptr_t)p & 15) == 0) {
        uint4 *p4 = reinterpret_cast<uint4 *>(p);
        for (int64_t e = start; e < n / 4; e += step) p4[e] = uint4{0u, 0u, 0u, 0u};
        for (int64_t e = n / 4 * 4 + start; e < n; e += step) p[e] = 0u;
    } else {
        for (int64_t e = start; e < n; e += step) p[e] = 0u;
    }
}

hipError_t launch_fill_zero(void *p, size_t bytes, hipStream_t st)
{
    if (bytes == 0) return hipSuccess;
    if (((uintptr_t)p & 3) != 0 || (bytes & 3) != 0) return hipErrorInvalidValue;
    const int64_t n = (int64_t)(bytes / 4);
    int64_t blocks = (n / 4 + kGenThreads - 1) / kGenThreads;
    blocks = blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks);
    LaunchCtx lc;
    lc.st = st;
    return launch(k_fill_zero, dim3((unsigned)blocks), dim3(kGenThreads), 0, lc, (uint32_t *)p, n);
}

// ---------------------------------------------------------------------------------------
// Averaging output units (Fig. 1): per stream and channel, the sum over all positions of the
// rows the last layer has completed, and the running mean.  One workgroup per (stream, block of
// 64 channels); four groups of lanes take every fourth position and are added in a fixed order.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_head_accumulate(const HeadAcc a, const StreamSel sel, int64_t first_slot,
                                                         int n_rows)
{
    __shared__ double part[4][64];
    const int stream = sel_stream(sel, blockIdx.z);
    const int cl = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int ch = blockIdx.x * 64 + cl;
    const uint32_t *src = (const uint32_t *)a.src + (int64_t)stream * a.src_stream_stride;
    double acc = 0.0;
    if (ch < a.c) {
        for (int r = 0; r < n_rows; ++r) {
            int64_t slot = first_slot + r;
            if (slot >= a.out_cap) slot -= a.out_cap;
            const uint32_t *row = src + slot * (int64_t)a.w * a.c;
            for (int x = grp; x < a.w; x += 4) {
                const uint32_t u = row[(int64_t)x * a.c + ch];
                acc += a.is_int ? (double)(int32_t)u : (double)__uint_as_float(u);
            }
        }
    }
    part[grp][cl] = acc;
    __syncthreads();
    if (grp == 0 && ch < a.c) {
        const int64_t at = (int64_t)stream * a.c + ch;
        double sum = a.zero_first ? 0.0 : a.sums[at];
        sum += ((part[0][cl] + part[1][cl]) + part[2][cl]) + part[3][cl];
        a.sums[at] = sum;
        a.mean[at] = a.count > 0.0 ? sum / a.count : 0.0;
    }
}

hipError_t launch_head_accumulate(const HeadAcc &a, const StreamSel &sel, int64_t first_slot, int n_rows,
                                  const LaunchCtx &lc)
{
    return launch(k_head_accumulate, dim3((unsigned)((a.c + 63) / 64), 1, sel.n), dim3(256), 0, lc, a, sel, first_slot,
                  n_rows);
}

// ---------------------------------------------------------------------------------------
// Fully connected output units (Sec. 4: the output units whose values settle as rows come in): every
// value of a completed row is an event that adds weight * value to each unit (Sec. 3, the same
// event-delivery rule one layer up; zero values are skipped).  One workgroup per (stream, unit);
// lanes stride over the rows' elements, partial sums are added in a fixed order.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_head_units(const HeadUnits a, const StreamSel sel, int64_t first_slot, int n_rows)
{
    __shared__ double part[256];
    const int stream = sel_stream(sel, blockIdx.z), unit = blockIdx.x;
    const uint32_t *src = (const uint32_t *)a.src + (int64_t)stream * a.src_stream_stride;
    const float *w = a.weights + (int64_t)unit * a.map_elems;
    const int64_t row_elems = (int64_t)a.w * a.c;
    double acc = 0.0;
    for (int r = 0; r < n_rows; ++r) {
        int64_t slot = first_slot + r;
        if (slot >= a.out_cap) slot -= a.out_cap;
        const uint32_t *row = src + slot * row_elems;
        const float *wr = w + (a.row0 + r) * row_elems;
        for (int64_t e = threadIdx.x; e < row_elems; e += 256) {
            const uint32_t u = row[e];
            const double v = a.is_int ? (double)(int32_t)u : (double)__uint_as_float(u);
            if (v != 0.0) acc += v * (double)wr[e];
        }
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const int64_t at = (int64_t)stream * a.n_units + unit;
        const double start = a.zero_first ? (a.bias ? (double)a.bias[unit] : 0.0) : a.values[at];
        a.values[at] = start + part[0];
    }
}

hipError_t launch_head_units(const HeadUnits &a, const StreamSel &sel, int64_t first_slot, int n_rows, const LaunchCtx &lc)
{
    return launch(k_head_units, dim3((unsigned)a.n_units, 1, sel.n), dim3(256), 0, lc, a, sel, first_slot, n_rows);
}

}  // namespace idf
