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
#include <cstdlib>

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
    static __device__ __forceinline__ t mac(t acc, t d, w_t w) { return acc + __mul24(d, (t)w); }     // differences of announced int8 values: well inside 24 bits
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

// 3x3 / stride 1 / padding 1 conv layers: the same update, laid out for the vector units.  A lane
// owns a chunk's output channel for POS neighbouring positions of every output row the segment's
// delta rows reach, and its cells stay in registers from the first delta to the announcement; a
// workgroup is one stream's row stretch of up to 256 / G lane groups.  The delta rows are staged
// in LDS, all input channels at once if they fit (else 16 at a time), as [row][channel][position],
// so that a lane reads the deltas its positions look at through one tap row as one or two wide
// reads of a single address per group; a weight is fetched once per lane and used for every cell
// it owns.  Zero deltas are multiplied like any other here: among the rows a segment's events
// reach, about half of the announced values change, and a multiply-add costs less than finding
// out.  (The sum of a cell is taken channel by channel, delta row by delta row: float results
// differ from k_eager_conv's in the last bits.)
//   k_eager_conv3x3_band: NIN delta rows, NIN + 2 output rows (those outside the map are worked out
//     and dropped), no test anywhere in the loop over the channels;
//   k_eager_conv3x3_rows: any band, eight output rows per workgroup, a bit test per (delta row, tap row).
constexpr int kEagLds = 60 * 1024;
// Input channels staged at a time: all of them when the staged rows fit the LDS budget, else 16.
__host__ __device__ inline int eager_chunk(int rows, int c_in, int xtp) { return (size_t)rows * c_in * xtp * 4 <= (size_t)kEagLds ? c_in : 16; }

// What a workgroup of either kernel knows about itself.
template <int P, int POS> struct EagerTile {
    using val_t = typename Val<P>::t;
    int tid, nt, G, XT, XTP, x0, gi, xb, co, co_c, W;
    bool co_ok;
    __device__ __forceinline__ EagerTile(const Geom &g)
    {
        tid = threadIdx.x; nt = blockDim.x;
        int g_log = 4;                                          // G = 16, 32 or 64 lanes: the channels of a chunk
        while ((1 << g_log) < g.c_out && g_log < 6) ++g_log;
        G = 1 << g_log;
        XT = (nt >> g_log) * POS;                               // positions per workgroup
        XTP = (XT + 2 + 3) & ~3;                                // a staged row: one position of halo either side, 16-byte rows
        const int co_chunks = (g.c_out + G - 1) >> g_log;
        const int x_tile = blockIdx.x / co_chunks, chunk = blockIdx.x - x_tile * co_chunks;
        x0 = x_tile * XT;
        gi = tid >> g_log;
        xb = x0 + gi * POS;
        co = chunk * G + (tid & (G - 1));
        co_ok = co < g.c_out;
        co_c = co_ok ? co : g.c_out - 1;
        W = g.w_out;                                            // = g.w_in
    }
    // n_rows delta rows from row i_first on go to LDS rows lds_row0 .. as [row][channel][position], channels [ci0, ci0 + ck)
    __device__ __forceinline__ void stage(const EagerStep &a, const val_t *din, val_t *lds, int i_first, int n_rows, int lds_row0, int ckm, int ci0, int ck) const
    {
        typedef val_t v4 __attribute__((ext_vector_type(4)));
        const Geom &g = a.g;
        const int spots = n_rows * (XT + 2);                    // (row, position) of the staged stretch
        for (int i = tid; i < spots; i += nt) {
            const int r = i / (XT + 2), xi = i - r * (XT + 2);
            const int x = x0 - 1 + xi;
            const bool in = x >= 0 && x < W;
            const val_t *src = din + ((int64_t)((i_first + r) % a.in_rows) * W + (in ? x : 0)) * g.c_in + ci0;
            val_t *dst = lds + ((lds_row0 + r) * ckm) * XTP + xi;
            if ((ck & 15) == 0 && (g.c_in & 3) == 0) {
                for (int q0 = 0; q0 < ck; q0 += 16) {
                    v4 v[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const v4 *>(src + q0 + 4 * q);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if (!in) v[q] = v4{0, 0, 0, 0};
                        val_t *d4 = dst + (q0 + 4 * q) * XTP;
                        d4[0] = v[q].x; d4[XTP] = v[q].y; d4[2 * XTP] = v[q].z; d4[3 * XTP] = v[q].w;
                    }
                }
            } else {
                for (int cc = 0; cc < ck; ++cc) dst[cc * XTP] = in ? src[cc] : (val_t)0;
            }
        }
    }
    // the POS + 2 deltas this lane's positions look at in one staged row of one channel
    __device__ __forceinline__ void window(const val_t *wp, val_t (&win)[POS + 2]) const
    {
        typedef val_t v4 __attribute__((ext_vector_type(4)));
        typedef val_t v2 __attribute__((ext_vector_type(2)));
        if (POS == 2) {                               // two positions: the window starts on an 8-byte boundary only
            const v2 q0 = *reinterpret_cast<const v2 *>(wp), q1 = *reinterpret_cast<const v2 *>(wp + 2);
            win[0] = q0.x; win[1] = q0.y; win[2] = q1.x; win[3] = q1.y;
            return;
        }
        const v4 q0 = *reinterpret_cast<const v4 *>(wp);
        win[0] = q0.x; win[1] = q0.y; win[2] = q0.z; win[3] = q0.w;
        if (POS == 8) {
            const v4 q1 = *reinterpret_cast<const v4 *>(wp + 4);
            win[4] = q1.x; win[5] = q1.y; win[6] = q1.z; win[7] = q1.w;
        }
        const v2 q2 = *reinterpret_cast<const v2 *>(wp + POS);
        win[POS] = q2.x; win[POS + 1] = q2.y;
    }
};

// Rows o_first .. o_first + ROWS - 1 of the lane's cells (bit j of rows_on: row j exists and belongs to
// this workgroup): the state as it was, or zero / the bias where it starts.
template <int P, int ROWS, int POS>
__device__ __forceinline__ void eager_load_state(const EagerStep &a, const EagerTile<P, POS> &t, int stream, int o_first, unsigned int rows_on,
                                                 typename Val<P>::t (&acc)[ROWS][POS])
{
    using val_t = typename Val<P>::t;
    const Geom &g = a.g;
    const val_t bias_v = a.init_bias && a.bias ? ((const val_t *)a.bias)[t.co_c] : (val_t)0;
    const val_t *c_old = (const val_t *)a.c + (int64_t)stream * a.c_stride;
    const int64_t row_elems = (int64_t)t.W * g.c_out;
    int slot = (o_first % a.c_rows + a.c_rows) % a.c_rows;      // (o_first may be -1: the row above the map)
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const int o = o_first + j;
        const bool keep = ((rows_on >> j) & 1u) && !a.init_bias && o < a.fresh_lo && t.co_ok;    // a row reached before: its state continues
#pragma unroll
        for (int p = 0; p < POS; ++p) {
            acc[j][p] = bias_v;
            if (keep && t.xb + p < t.W) acc[j][p] = c_old[(int64_t)slot * row_elems + (int64_t)(t.xb + p) * g.c_out + t.co];
        }
        slot = slot + 1 == a.c_rows ? 0 : slot + 1;
    }
}

// The same rows go back; every cell announces f(c) minus what it announced last.  What was announced
// is asked for first, for all cells at once: taken cell by cell between the stores, every request
// would wait out a memory round trip of its own.  Returns this lane's events.
template <int P, int ROWS, int POS>
__device__ __forceinline__ unsigned int eager_announce(const EagerStep &a, const EagerTile<P, POS> &t, int stream, int o_first, unsigned int rows_on,
                                                       const typename Val<P>::t (&acc)[ROWS][POS])
{
    using V = Val<P>;
    using val_t = typename V::t;
    const Geom &g = a.g;
    val_t *c_new = (val_t *)a.c + (int64_t)stream * a.c_stride;
    val_t *ann = (val_t *)a.ann + (int64_t)stream * a.ann_stride;
    val_t *dlt = (val_t *)a.dlt_out + (int64_t)stream * a.dlt_stride;
    const int64_t row_elems = (int64_t)t.W * g.c_out;
    uint32_t cell[POS];
    bool have[POS];
#pragma unroll
    for (int p = 0; p < POS; ++p) {
        have[p] = t.co_ok && t.xb + p < t.W;
        cell[p] = (uint32_t)((have[p] ? t.xb + p : 0) * g.c_out + t.co_c);
    }
    val_t old[ROWS][POS];
    int slot = (o_first % a.ann_rows + a.ann_rows) % a.ann_rows;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const bool first = o_first + j >= a.fresh_lo && !a.init_bias;           // nothing announced so far
        const bool on = ((rows_on >> j) & 1u) && !first;
#pragma unroll
        for (int p = 0; p < POS; ++p) {
            old[j][p] = 0;
            if (on && have[p]) old[j][p] = ann[(int64_t)slot * row_elems + cell[p]];
        }
        slot = slot + 1 == a.ann_rows ? 0 : slot + 1;
    }
    unsigned int events = 0;
    int s_c = (o_first % a.c_rows + a.c_rows) % a.c_rows, s_d = (o_first % a.dlt_rows + a.dlt_rows) % a.dlt_rows;
    slot = (o_first % a.ann_rows + a.ann_rows) % a.ann_rows;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        if ((rows_on >> j) & 1u) {
#pragma unroll
            for (int p = 0; p < POS; ++p) {
                if (!have[p]) continue;
                c_new[(int64_t)s_c * row_elems + cell[p]] = acc[j][p];
                const val_t h = V::act(g, acc[j][p], a.round_bf16), d = h - old[j][p];
                ann[(int64_t)slot * row_elems + cell[p]] = h;
                dlt[(int64_t)s_d * row_elems + cell[p]] = d;
                events += d != 0;
            }
        }
        s_c = s_c + 1 == a.c_rows ? 0 : s_c + 1;
        s_d = s_d + 1 == a.dlt_rows ? 0 : s_d + 1;
        slot = slot + 1 == a.ann_rows ? 0 : slot + 1;
    }
    return events;
}

// The workgroup's events: one addition to the stream's counter of the next layer.
__device__ __forceinline__ void eager_count(const EagerStep &a, int stream, unsigned int events, unsigned int *ev_sum)
{
    if (!a.stats || a.layer + 1 >= a.n_layers) return;
    __syncthreads();
    if (events) atomicAdd(ev_sum, events);
    __syncthreads();
    if (threadIdx.x == 0 && *ev_sum) atomicAdd(a.stats + ((int64_t)stream * a.n_layers + a.layer + 1) * 2, (unsigned long long)*ev_sum);
}

template <int P, int NIN, int POS>
__global__ void __launch_bounds__(256) k_eager_conv3x3_band(const EagerStep a, const StreamSel sel)
{
    using V = Val<P>;
    using val_t = typename V::t;
    using w_t = typename V::w_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char eag_smem[];
    val_t *lds = reinterpret_cast<val_t *>(eag_smem);
    __shared__ unsigned int ev_sum;
    const Geom &g = a.g;
    const int stream = sel_stream(sel, blockIdx.z);
    const EagerTile<P, POS> t(g);
    if (t.tid == 0) ev_sum = 0;
    // delta rows [i_lo, i_lo + NIN) reach output rows i_lo - 1 .. i_lo + NIN: row j of the lane's cells is row i_lo - 1 + j
    const int o_first = a.i_lo - 1;
    unsigned int rows_on = 0;
#pragma unroll
    for (int j = 0; j < NIN + 2; ++j)
        if (o_first + j >= a.o_lo && o_first + j < a.o_hi) rows_on |= 1u << j;
    rows_on = __builtin_amdgcn_readfirstlane(rows_on);
    val_t acc[NIN + 2][POS];
    eager_load_state<P, NIN + 2, POS>(a, t, stream, o_first, rows_on, acc);

    const val_t *din = (const val_t *)a.dlt_in + (int64_t)stream * a.in_map_stride;
    // this lane's nine weights of an input channel: byte offsets from a base that moves on channel by channel
    uint32_t woff[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) woff[k] = (uint32_t)(((size_t)k * g.c_in * g.c_out + t.co_c) * sizeof(w_t));
    const uint32_t w_step = (uint32_t)(g.c_out * sizeof(w_t));
    auto weight = [&](const unsigned char *base, int k) { return *reinterpret_cast<const w_t *>(base + woff[k]); };
    const int ckm = eager_chunk(NIN, g.c_in, t.XTP);
    for (int ci0 = 0; ci0 < g.c_in; ci0 += ckm) {
        const int ck = g.c_in - ci0 < ckm ? g.c_in - ci0 : ckm;
        __syncthreads();                                        // the chunk before has been read by every lane
        t.stage(a, din, lds, a.i_lo, NIN, 0, ckm, ci0, ck);
        __syncthreads();
        const unsigned char *wb = (const unsigned char *)a.w + (size_t)ci0 * w_step;
        w_t wn[9];                                              // the next channel's weights are on their way while this one's are used
#pragma unroll
        for (int k = 0; k < 9; ++k) wn[k] = weight(wb, k);
        const val_t *lrow = lds + t.gi * POS;
        for (int cc = 0; cc < ck; ++cc) {
            w_t wv[9];
            if (cc + 1 < ck) wb += w_step;
#pragma unroll
            for (int k = 0; k < 9; ++k) { wv[k] = wn[k]; wn[k] = weight(wb, k); }
#pragma unroll
            for (int r = 0; r < NIN; ++r) {
                val_t win[POS + 2];
                t.window(lrow + (r * ckm + cc) * t.XTP, win);
#pragma unroll
                for (int ky = 0; ky < 3; ++ky)                  // delta row i_lo + r is what row i_lo + r + 1 - ky sees through tap row ky
#pragma unroll
                    for (int kx = 0; kx < 3; ++kx)
#pragma unroll
                        for (int p = 0; p < POS; ++p) acc[r + 2 - ky][p] = V::mac(acc[r + 2 - ky][p], win[p + kx], wv[ky * 3 + kx]);
            }
        }
    }
    const unsigned int events = eager_announce<P, NIN + 2, POS>(a, t, stream, o_first, rows_on, acc);
    eager_count(a, stream, events, &ev_sum);
}

template <int P, int POS>
__global__ void __launch_bounds__(256) k_eager_conv3x3_rows(const EagerStep a, const StreamSel sel)
{
    constexpr int R = 8;
    using V = Val<P>;
    using val_t = typename V::t;
    using w_t = typename V::w_t;
    extern __shared__ __attribute__((aligned(16))) unsigned char eag_smem[];
    val_t *lds = reinterpret_cast<val_t *>(eag_smem);
    __shared__ unsigned int ev_sum;
    const Geom &g = a.g;
    const int stream = sel_stream(sel, blockIdx.z);
    const EagerTile<P, POS> t(g);
    if (t.tid == 0) ev_sum = 0;
    const int oa = a.o_lo + blockIdx.y * R;
    const int nr = (a.o_hi - oa) < R ? (a.o_hi - oa) : R;
    // the delta rows of the layer before that reach rows [oa, oa + nr)
    const int ia = oa - 1 > a.i_lo ? oa - 1 : a.i_lo;
    const int ib = oa + nr + 1 < a.i_hi ? oa + nr + 1 : a.i_hi;
    const int n_in = ib > ia ? ib - ia : 0;
    const unsigned int rows_on = __builtin_amdgcn_readfirstlane((1u << nr) - 1u);
    val_t acc[R][POS];
    eager_load_state<P, R, POS>(a, t, stream, oa, rows_on, acc);
    // which (delta row, tap row) pairs exist for this workgroup: bit ri * 3 + ky, delta row oa - 1 + ri
    // seen by output row oa + ri - ky
    unsigned int pairs_on = 0;
#pragma unroll
    for (int ri = 0; ri < R + 2; ++ri)
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int iy = oa - 1 + ri, rr = ri - ky;
            if (iy >= ia && iy < ib && rr >= 0 && rr < nr) pairs_on |= 1u << (ri * 3 + ky);
        }
    pairs_on = __builtin_amdgcn_readfirstlane(pairs_on);        // one scalar word: a bit test and a scalar branch per pair

    const val_t *din = (const val_t *)a.dlt_in + (int64_t)stream * a.in_map_stride;
    uint32_t woff[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) woff[k] = (uint32_t)(((size_t)k * g.c_in * g.c_out + t.co_c) * sizeof(w_t));
    const uint32_t w_step = (uint32_t)(g.c_out * sizeof(w_t));
    auto weight = [&](const unsigned char *base, int k) { return *reinterpret_cast<const w_t *>(base + woff[k]); };
    const int ckm = eager_chunk(R + 2, g.c_in, t.XTP);
    for (int ci0 = 0; ci0 < g.c_in && n_in > 0; ci0 += ckm) {
        const int ck = g.c_in - ci0 < ckm ? g.c_in - ci0 : ckm;
        __syncthreads();                                        // the chunk before has been read by every lane
        t.stage(a, din, lds, ia, n_in, ia - (oa - 1), ckm, ci0, ck);            // a row is staged by its place among the R + 2
        __syncthreads();
        const unsigned char *wb = (const unsigned char *)a.w + (size_t)ci0 * w_step;
        w_t wn[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) wn[k] = weight(wb, k);
        const val_t *lrow = lds + t.gi * POS;
        for (int cc = 0; cc < ck; ++cc) {
            w_t wv[9];
            if (cc + 1 < ck) wb += w_step;
#pragma unroll
            for (int k = 0; k < 9; ++k) { wv[k] = wn[k]; wn[k] = weight(wb, k); }
            // (kept from being tested once and for all outside the loop: some thirty lane masks held in scalar registers
            // across it cost more, spilled and reloaded, than a bit test per pair)
            unsigned int on = pairs_on;
            asm volatile("" : "+s"(on));
#pragma unroll
            for (int ri = 0; ri < R + 2; ++ri) {
                if (((on >> (ri * 3)) & 7u) == 0) continue;                     // the same for every lane
                val_t win[POS + 2];
                t.window(lrow + (ri * ckm + cc) * t.XTP, win);
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const int rr = ri - ky;                     // output row oa + rr looks at this delta row through tap row ky
                    if (rr < 0 || rr >= R) continue;
                    if (!((on >> (ri * 3 + ky)) & 1u)) continue;
#pragma unroll
                    for (int kx = 0; kx < 3; ++kx)
#pragma unroll
                        for (int p = 0; p < POS; ++p) acc[rr][p] = V::mac(acc[rr][p], win[p + kx], wv[ky * 3 + kx]);
                }
            }
        }
    }
    const unsigned int events = eager_announce<P, R, POS>(a, t, stream, oa, rows_on, acc);
    eager_count(a, stream, events, &ev_sum);
}

template <int P, int POS>
hipError_t launch_eager_band(int n_in, dim3 grid, dim3 block, size_t lds, const LaunchCtx &lc, const EagerStep &a, const StreamSel &sel)
{
    switch (n_in) {
    case 1: return launch(k_eager_conv3x3_band<P, 1, POS>, grid, block, lds, lc, a, sel);
    case 2: return launch(k_eager_conv3x3_band<P, 2, POS>, grid, block, lds, lc, a, sel);
    case 3: return launch(k_eager_conv3x3_band<P, 3, POS>, grid, block, lds, lc, a, sel);
    case 4: return launch(k_eager_conv3x3_band<P, 4, POS>, grid, block, lds, lc, a, sel);
    case 5: return launch(k_eager_conv3x3_band<P, 5, POS>, grid, block, lds, lc, a, sel);
    case 6: return launch(k_eager_conv3x3_band<P, 6, POS>, grid, block, lds, lc, a, sel);
    default: return hipErrorInvalidValue;
    }
}

template <int P>
hipError_t launch_eager_conv3x3(const EagerStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    const Geom &g = a.g;
    int G = 16;
    while (G < g.c_out && G < 64) G *= 2;
    const int rows = a.o_hi - a.o_lo, n_in = a.i_hi - a.i_lo;
    const int co_chunks = (g.c_out + G - 1) / G;
    // one workgroup for the whole band when it is what a short segment gives: up to six delta rows and exactly the rows they reach
    const int top = a.i_lo - 1 > 0 ? a.i_lo - 1 : 0, bottom = a.i_hi + 1 < g.h_out ? a.i_hi + 1 : g.h_out;
    const bool band = n_in >= 1 && n_in <= 6 && a.o_lo == top && a.o_hi == bottom;
    const int row_groups = band ? 1 : (rows + 7) / 8;
    // eight positions per lane reuse a weight for more cells; four or two give more waves while the launch is small
    // (measured on 256 streams of 32 x 32: 5.9 ms per batch with eight, 3.9 with four)
    auto waves = [&](int pos) { return (int64_t)row_groups * co_chunks * sel.n * (((int64_t)((g.w_out + pos - 1) / pos) * G + 63) / 64); };
    const char *force = getenv("IDF_EAGER_POS");               // "2", "4" or "8": for tests of the shape the sizes at hand would not pick
    const int pos = force ? (force[0] == '8' ? 8 : force[0] == '2' ? 2 : 4) : waves(8) >= 2048 ? 8 : waves(4) >= 2048 ? 4 : 2;
    int groups = (g.w_out + pos - 1) / pos;
    if (groups > 256 / G) groups = 256 / G;
    const int XT = groups * pos, x_tiles = (g.w_out + XT - 1) / XT, XTP = (XT + 2 + 3) & ~3;
    const int staged = band ? n_in : 10;
    const size_t lds = (size_t)staged * eager_chunk(staged, g.c_in, XTP) * XTP * 4;
    const dim3 grid((unsigned)(x_tiles * co_chunks), (unsigned)row_groups, sel.n), block((unsigned)(groups * G));
    if (band) return pos == 8 ? launch_eager_band<P, 8>(n_in, grid, block, lds, lc, a, sel) : pos == 4 ? launch_eager_band<P, 4>(n_in, grid, block, lds, lc, a, sel)
                                                                                                       : launch_eager_band<P, 2>(n_in, grid, block, lds, lc, a, sel);
    return pos == 8 ? launch(k_eager_conv3x3_rows<P, 8>, grid, block, lds, lc, a, sel) : pos == 4 ? launch(k_eager_conv3x3_rows<P, 4>, grid, block, lds, lc, a, sel)
                                                                                                   : launch(k_eager_conv3x3_rows<P, 2>, grid, block, lds, lc, a, sel);
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
        int G = 16;
        while (G < a.g.c_out && G < 64) G *= 2;
        const Geom &g = a.g;
        // Float nets take the register-tiled kernels, which multiply every delta of the band.  The quantised nets stay with
        // the kernel below that visits the non-zero deltas only: announced values clamped to a few levels change rarely
        // (a tenth of the deltas are events on the int8 workload, where it is the faster of the two in the deep layers),
        // unless IDF_EAGER_TILED asks otherwise; IDF_EAGER_PLAIN sends every net there.
        const bool tiled = g.k_h == 3 && g.k_w == 3 && g.s_h == 1 && g.s_w == 1 && g.p_h == 1 && g.p_w == 1 && !getenv("IDF_EAGER_PLAIN");
        if (tiled && prec == IDF_PREC_I8 && getenv("IDF_EAGER_TILED")) return launch_eager_conv3x3<kI8>(a, sel, lc);
        if (tiled && prec == IDF_PREC_BF16) return launch_eager_conv3x3<kBf16>(a, sel, lc);
        if (tiled && prec == IDF_PREC_F32) return launch_eager_conv3x3<kF32>(a, sel, lc);
        // a group of G lanes per (position, chunk of G channels): see k_eager_conv
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
