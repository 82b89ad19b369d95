// Eager emission (Sec. 3, the stateful neuron and the event definition taken literally): every
// neuron keeps its state c and the value it last announced; whenever f(c) differs from that
// value the difference goes out as an event at once, is added, weighted, into the state of the
// neurons it connects to, and those may announce changes in turn.  Nothing waits for a row to be
// complete, so after any pushed segment the announced activations of every layer are those of the
// conventional network applied to the input seen so far, the rest taken as zero (Sec. 4, Fig. 3:
// the output is updated with every row presented).
//
// On the GPU the events of one segment are delivered layer by layer as a band of delta rows:
// each cell of the band a layer can reach gathers w * delta over its footprint inside the band
// of the layer before (zero deltas are skipped), announces f(c) minus what it announced last, and
// writes that difference into its own delta band.  A max-pool is a stateful node that
// re-evaluates its window of announced values.  Per stream and level the rows that can still
// change or be looked at are kept in a ring (row r in slot r mod rows kept: the cone of Sec. 3),
// or every row when the net has biases; a row reached for the first time starts from zero
// whatever its slot held.  All values are 4 bytes: float32, or int32 for the quantised nets; a
// bfloat16 net announces values rounded to bfloat16 (the last layer unrounded).
#include "idf.h"
#include "idf_kernels.h"

namespace idf {

namespace {

enum { kF32 = 0, kI8 = 1, kBf16 = 2 };

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

template <int P> struct Val;
template <> struct Val<kF32> {
    using t = float; using w_t = float; using in_t = float;
    static __device__ __forceinline__ t from_in(in_t v) { return v; }
    static __device__ __forceinline__ t act(const Geom &g, t c, int) { return g.act == IDF_ACT_NONE ? c : fmaxf(c, 0.f); }
    static __device__ __forceinline__ t mac(t acc, t d, w_t w) { return fmaf(d, w, acc); }
};
template <> struct Val<kBf16> {
    using t = float; using w_t = uint16_t; using in_t = uint16_t;
    static __device__ __forceinline__ t from_in(in_t v) { return bf16_bits_to_float(v); }
    static __device__ __forceinline__ t act(const Geom &g, t c, int round)
    {
        const t h = g.act == IDF_ACT_NONE ? c : fmaxf(c, 0.f);
        return round ? (t)(__bf16)h : h;                        // to nearest, ties to even
    }
    static __device__ __forceinline__ t mac(t acc, t d, w_t w) { return fmaf(d, bf16_bits_to_float(w), acc); }
};
template <> struct Val<kI8> {
    using t = int32_t; using w_t = int8_t; using in_t = int8_t;
    static __device__ __forceinline__ t from_in(in_t v) { return v; }
    static __device__ __forceinline__ t act(const Geom &g, t c, int)
    {
        if (g.act == IDF_ACT_NONE) return c;
        t r = c > 0 ? c : 0;
        if (g.act == IDF_ACT_RELU_SHR_CLAMP) { r >>= g.shr; r = r > g.clamp_hi ? g.clamp_hi : r; }
        return r;
    }
    static __device__ __forceinline__ t mac(t acc, t d, w_t w) { return acc + d * (t)w; }
};

// Non-zero differences announced by this workgroup: the events delivered to the next layer.
__device__ __forceinline__ void count_events(bool nz, unsigned long long *dst)
{
    const unsigned long long b = __ballot(nz);
    if (dst && b && (threadIdx.x & 63) == 0) atomicAdd(dst, (unsigned long long)__popcll(b));
}

// The pushed rows become the announced input; what changed goes out as the input's events.
template <int P>
__global__ void __launch_bounds__(256) k_eager_input(const EagerStep a, const StreamSel sel)
{
    using V = Val<P>;
    using val_t = typename V::t;
    const int stream = sel_stream(sel, blockIdx.z);
    const int64_t row_elems = (int64_t)a.w_out * a.c_out, n = (int64_t)(a.o_hi - a.o_lo) * row_elems;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool nz = false;
    if (i < n) {
        const typename V::in_t *in = (const typename V::in_t *)a.in + (int64_t)(sel.pos0 + blockIdx.z) * a.in_stream_stride;
        const int row = a.o_lo + (int)(i / row_elems);
        const int64_t col = i - (int64_t)(row - a.o_lo) * row_elems;
        val_t *ann = (val_t *)a.ann + (int64_t)stream * a.ann_stride + (int64_t)(row % a.ann_rows) * row_elems + col;
        val_t *dlt = (val_t *)a.dlt_out + (int64_t)stream * a.dlt_stride + (int64_t)(row % a.dlt_rows) * row_elems + col;
        const val_t v = V::from_in(in[i]), d = v - (row >= a.fresh_lo ? (val_t)0 : *ann);
        *ann = v; *dlt = d;
        nz = d != 0;
    }
    count_events(nz, a.stats ? a.stats + ((int64_t)stream * a.n_layers + a.layer) * 2 : nullptr);
}

// Conv layer: cells of output rows [o_lo, o_hi) take in the delta rows [i_lo, i_hi) of the layer before.
// A group of G lanes (G = c_out rounded up to a power of two, at most 64) owns one position and a
// chunk of G output channels, one cell per lane.  For each tap the group reads the delta vector of the
// position it looks at once, G input channels at a time, one value per lane; a ballot of the
// non-zero values is the list of events, and only those are visited: the value comes from the lane
// that holds it, the weight from memory, one multiply-add per cell.  A zero costs nothing but its
// share of that one read.  The order of the additions is that of the footprint (ky, kx, channel).
template <int P>
__global__ void __launch_bounds__(256) k_eager_conv(const EagerStep a, const StreamSel sel)
{
    using V = Val<P>;
    using val_t = typename V::t;
    const Geom &g = a.g;
    const int stream = sel_stream(sel, blockIdx.z);
    const int lane = threadIdx.x & 63;
    int g_log = 4;                                              // G = 16, 32 or 64
    while ((1 << g_log) < g.c_out && g_log < 6) ++g_log;
    const int G = 1 << g_log, per_wave = 64 >> g_log;
    const int grp = lane >> g_log, col = lane & (G - 1);
    const int co_chunks = (g.c_out + G - 1) >> g_log;
    const int64_t units = (int64_t)(a.o_hi - a.o_lo) * g.w_out * co_chunks;      // (position, channel chunk)
    const int64_t unit = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * per_wave + grp;
    const bool have = unit < units;
    const int64_t u = have ? unit : units - 1;                  // clamped: every lane stays in the loops
    const int chunk = (int)(u % co_chunks);
    const int64_t pos = u / co_chunks;
    const int x = (int)(pos % g.w_out), o = a.o_lo + (int)(pos / g.w_out);
    const int co = chunk * G + col;
    const bool mine = have && co < g.c_out;
    const int co_c = co < g.c_out ? co : g.c_out - 1;
    const val_t *din = (const val_t *)a.dlt_in + (int64_t)stream * a.in_map_stride;
    const typename V::w_t *w = (const typename V::w_t *)a.w;
    const int64_t in_row = (int64_t)x * g.c_out + co_c;         // cell within its row
    const int64_t c_cell = (int64_t)stream * a.c_stride + (int64_t)(o % a.c_rows) * g.w_out * g.c_out + in_row;
    const int64_t ann_cell = (int64_t)stream * a.ann_stride + (int64_t)(o % a.ann_rows) * g.w_out * g.c_out + in_row;
    const int64_t dlt_cell = (int64_t)stream * a.dlt_stride + (int64_t)(o % a.dlt_rows) * g.w_out * g.c_out + in_row;
    const bool fresh = o >= a.fresh_lo;                         // reached for the first time: starts from zero
    val_t c = a.init_bias ? (a.bias ? ((const val_t *)a.bias)[co_c] : (val_t)0) : (fresh ? (val_t)0 : ((val_t *)a.c)[c_cell]);
    const unsigned long long gbits = G == 64 ? ~0ull : ((1ull << G) - 1ull);
    for (int ky = 0; ky < g.k_h; ++ky) {
        const int iy = o * g.s_h - g.p_h + ky;
        const bool row_ok = iy >= a.i_lo && iy < a.i_hi;        // only the rows that carry this segment's events
        for (int kx = 0; kx < g.k_w; ++kx) {
            const int ix = x * g.s_w - g.p_w + kx;
            const bool tap_ok = row_ok && ix >= 0 && ix < g.w_in;
            if (__ballot(tap_ok) == 0ull) continue;
            const val_t *dp = din + ((int64_t)((tap_ok ? iy : a.i_lo) % a.in_rows) * g.w_in + (tap_ok ? ix : 0)) * g.c_in;
            const typename V::w_t *wp = w + ((int64_t)(ky * g.k_w + kx) * g.c_in) * g.c_out + co_c;
            for (int j0 = 0; j0 < g.c_in; j0 += G) {
                const val_t dv = (tap_ok && j0 + col < g.c_in) ? dp[j0 + col] : (val_t)0;
                const unsigned long long all = __ballot(dv != 0);
                if (all == 0ull) continue;
                unsigned long long ev = (all >> (grp << g_log)) & gbits;    // this group's events
                while (__ballot(ev != 0ull) != 0ull) {
                    // four events at a time: their values and weights are all asked for before
                    // the first is used (a slot past the last event repeats the last one, adding nothing)
                    constexpr int kE = 4;
                    val_t d[kE];
                    typename V::w_t wv[kE];
                    int bit = 0;
#pragma unroll
                    for (int e = 0; e < kE; ++e) {
                        const bool on = ev != 0ull;
                        bit = on ? __builtin_ctzll(ev) : bit;
                        const val_t dd = __shfl(dv, (grp << g_log) + bit);
                        d[e] = on ? dd : (val_t)0;
                        wv[e] = wp[(int64_t)(j0 + bit) * g.c_out];
                        ev &= ev - 1ull;
                    }
#pragma unroll
                    for (int e = 0; e < kE; ++e)
                        if (d[e] != 0) c = V::mac(c, d[e], wv[e]);
                }
            }
        }
    }
    bool nz = false;
    if (mine) {
        ((val_t *)a.c)[c_cell] = c;
        const val_t h = V::act(g, c, a.round_bf16), d = h - (fresh && !a.init_bias ? (val_t)0 : ((val_t *)a.ann)[ann_cell]);
        ((val_t *)a.ann)[ann_cell] = h;
        ((val_t *)a.dlt_out)[dlt_cell] = d;
        nz = d != 0;
    }
    count_events(nz, a.stats && a.layer + 1 < a.n_layers ? a.stats + ((int64_t)stream * a.n_layers + a.layer + 1) * 2 : nullptr);
}

// 2x2 max-pool as a stateful node: re-evaluates its window of announced values.
template <int P>
__global__ void __launch_bounds__(256) k_eager_pool(const EagerStep a, const StreamSel sel)
{
    using val_t = typename Val<P>::t;
    const Geom &g = a.g;
    const int stream = sel_stream(sel, blockIdx.z);
    const int64_t n = (int64_t)(a.o_hi - a.o_lo) * g.w_out * g.c_out;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    bool nz = false;
    if (i < n) {
        const int ch = (int)(i % g.c_out);
        const int64_t pos = i / g.c_out;
        const int x = (int)(pos % g.w_out), o = a.o_lo + (int)(pos / g.w_out);
        const val_t *ain = (const val_t *)a.ann_in + (int64_t)stream * a.in_map_stride;
        // a row of the window that has not been reached yet announces zero (the net starts from zero state)
        bool first = true;
        val_t m = 0;
        for (int dy = 0; dy < 2; ++dy)
            for (int dx = 0; dx < g.k_w; ++dx) {
                const int r = 2 * o + dy;
                const val_t v = r >= a.in_hi ? (val_t)0 : ain[((int64_t)(r % a.in_rows) * g.w_in + x * g.s_w + dx) * g.c_out + ch];
                m = (first || v > m) ? v : m;
                first = false;
            }
        const int64_t in_row = (int64_t)x * g.c_out + ch;
        const int64_t ann_cell = (int64_t)stream * a.ann_stride + (int64_t)(o % a.ann_rows) * g.w_out * g.c_out + in_row;
        const int64_t dlt_cell = (int64_t)stream * a.dlt_stride + (int64_t)(o % a.dlt_rows) * g.w_out * g.c_out + in_row;
        const val_t d = m - (o >= a.fresh_lo && !a.init_bias ? (val_t)0 : ((val_t *)a.ann)[ann_cell]);
        ((val_t *)a.ann)[ann_cell] = m;
        ((val_t *)a.dlt_out)[dlt_cell] = d;
        nz = d != 0;
    }
    count_events(nz, a.stats && a.layer + 1 < a.n_layers ? a.stats + ((int64_t)stream * a.n_layers + a.layer + 1) * 2 : nullptr);
}

}  // namespace

hipError_t launch_eager(int prec, int what, const EagerStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    const int64_t n = (int64_t)(a.o_hi - a.o_lo) * (what == 0 ? (int64_t)a.w_out * a.c_out : (int64_t)a.g.w_out * a.g.c_out);
    if (n <= 0) return hipSuccess;
    dim3 grid((unsigned)((n + 255) / 256), 1, sel.n);
    const dim3 block(256);
    if (what == 1) {
        // a group of G lanes per (position, chunk of G channels): see k_eager_conv
        int G = 16;
        while (G < a.g.c_out && G < 64) G *= 2;
        const int64_t units = (int64_t)(a.o_hi - a.o_lo) * a.g.w_out * ((a.g.c_out + G - 1) / G);
        const int per_block = 4 * (64 / G);
        grid.x = (unsigned)((units + per_block - 1) / per_block);
    }
    if (prec == IDF_PREC_I8) {
        if (what == 0) return launch(k_eager_input<kI8>, grid, block, 0, lc, a, sel);
        if (what == 1) return launch(k_eager_conv<kI8>, grid, block, 0, lc, a, sel);
        return launch(k_eager_pool<kI8>, grid, block, 0, lc, a, sel);
    }
    if (prec == IDF_PREC_BF16) {
        if (what == 0) return launch(k_eager_input<kBf16>, grid, block, 0, lc, a, sel);
        if (what == 1) return launch(k_eager_conv<kBf16>, grid, block, 0, lc, a, sel);
        return launch(k_eager_pool<kBf16>, grid, block, 0, lc, a, sel);
    }
    if (what == 0) return launch(k_eager_input<kF32>, grid, block, 0, lc, a, sel);
    if (what == 1) return launch(k_eager_conv<kF32>, grid, block, 0, lc, a, sel);
    return launch(k_eager_pool<kF32>, grid, block, 0, lc, a, sel);
}

}  // namespace idf
