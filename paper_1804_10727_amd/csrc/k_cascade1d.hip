// Depth-first cascade for 1-D nets: one launch per push, one workgroup per stream, every
// layer the segment can influence handled in turn (Sec. 3 first paragraph: each segment goes
// through all of the network it can influence before the next is looked at).
//
// The stream's whole retained state -- the rolling buffer of K rows of pre-activations c of
// every layer (Fig. 1) -- is brought into LDS when the kernel starts, lives there while the
// segment runs through the layers, and is written back once at the end.  Per layer the
// workgroup
//   1. has the new input rows in LDS, stored per input channel ([channel][row]) so that one
//      wide LDS read brings all new rows of a channel;
//   2. accumulates w * dh (event-delivery rule of Sec. 3) with output channels across lanes
//      and the input channels dealt round-robin to groups of lanes.  Zero values are not
//      events: a channel that is silent in every new row is skipped, and in short segments
//      single zero rows are branched over as well.  Each lane keeps the partial sums of all
//      touched output rows of its channel in registers; the register holding (input row j,
//      tap ky) is fixed at compile time;
//   3. adds the groups' partial sums in a fixed order to the retained c (or to the bias for
//      rows touched for the first time), then either activates and emits the row to the next
//      layer (LDS) -- counting the non-zero values it emits with a wave ballot, they are the
//      next layer's events -- or stores it back into the LDS copy of the rolling buffer.
//
// The kernel is a chain of dependent layers on one compute unit, and what limits it is the
// path from memory: every weight is needed exactly once per push and has to come through the
// vector memory pipeline of that one compute unit.  Hence the weights are one continuous
// stream of requests running four input channels ahead of their use, across layer boundaries
// (the tail of layer l already requests the head of layer l+1); the argument block is copied
// to LDS in one sweep; and nothing is stored to global memory before the last layer is done
// (loads, stores and atomics of a wave share one in-order counter here, so a store in the middle
// of the chain would make every later load wait for the store's acknowledgement).
//
// Serves float32 nets whose layers are all convolutions over a width-1 signal with at most 64
// channels, kernel height <= 9, stride <= 2 and at most 16 rows per layer per push.  Weights
// come packed [c_in][c_out][12 taps, zero padded]: three 16-byte loads per channel pair.
#include "idf.h"
#include "idf_kernels.h"

namespace idf {

namespace {

constexpr int kT = kCasThreads;
constexpr int kKMax = kCasKMax;
constexpr int kRowsMax = kCasRowsMax;
constexpr int kTMax = kRowsMax + kKMax - 1;          // touched output rows at most
constexpr int kCellsPerThread = (kTMax * 64 + kT - 1) / kT;
constexpr int kXStride = 20;                         // floats per channel in LDS (16 rows + pad, 16-byte aligned)
constexpr int kAhead = 4;                            // input channels whose weights are in flight
constexpr int kArgWords = (sizeof(CascadeArgs) + 3) / 4;
constexpr int kRingPerLayer = kKMax * 64;            // floats of rolling buffer per layer at most

constexpr int ceil_div_c(int a, int b) { return a >= 0 ? (a + b - 1) / b : -((-a) / b); }
// Offset of accumulator slot 0 relative to floor((y0+p)/S), and number of slots.
template <int S, int RHO> constexpr int slot_off() { return ceil_div_c(RHO - kKMax + 1, S); }
template <int S, int NIN, int RHO> constexpr int slot_cnt() { return (RHO + NIN - 1) / S - slot_off<S, RHO>() + 1; }

struct Lds {
    float x[2][64 * kXStride];                   // input rows of the current / next layer, [channel][row]
    float red[kT * kTMax];                       // partial sums [group][slot][channel lane]
    float ring[kCasMaxLayers][kRingPerLayer];    // the stream's rolling buffers, [layer][slot][channel]
    float bias[kCasMaxLayers][64];
    unsigned int events[kCasMaxLayers], taps[kCasMaxLayers];
    uint32_t args[kArgWords];                    // the kernel's argument block
};

// Pointers read back from LDS have lost their address space; saying "global" again lets the
// compiler use global (not flat) loads, whose completion order it can count on.
typedef __attribute__((address_space(1))) float gfloat;
template <class P> __device__ __forceinline__ const gfloat *as_global(const P *p) { return (const gfloat *)p; }

struct Wq { float w[kAhead][kCasTapsPad]; };     // weights of kAhead input channels, all taps

// Where a lane finds its weights of one layer: w[ci][co][taps] with ci = grp, grp + n_grp, ...
struct WSrc {
    const gfloat *w;
    int c_in, c_out, grp, n_grp, co_c, n_qp;     // n_qp: channels per lane, rounded up to kAhead
};

template <int NIN> __device__ __forceinline__ void load_rows(const float *p, float (&xv)[NIN])
{
#pragma unroll
    for (int q = 0; q < NIN / 4; ++q) {
        const float4 v = *reinterpret_cast<const float4 *>(p + 4 * q);
        xv[4 * q] = v.x; xv[4 * q + 1] = v.y; xv[4 * q + 2] = v.z; xv[4 * q + 3] = v.w;
    }
}

// Lane mapping of one layer: channel lane within the power-of-two pad of c_out, group of lanes.
struct Lanes { int cp_log, cp, co, grp, n_grp; };
__device__ __forceinline__ Lanes lanes_of(int cp_log, int tid)
{
    Lanes m;
    m.cp_log = cp_log; m.cp = 1 << cp_log;
    m.co = tid & (m.cp - 1); m.grp = tid >> cp_log; m.n_grp = kT >> cp_log;
    return m;
}

__device__ __forceinline__ WSrc wsrc_of(const CascadeArgs &a, int l, int tid)
{
    const Lanes m = lanes_of(a.sched[l].cp_log, tid);
    WSrc s;
    s.w = as_global((const float *)a.w[l]);
    s.c_in = a.g[l].c_in; s.c_out = a.g[l].c_out;
    s.grp = m.grp; s.n_grp = m.n_grp;
    s.co_c = m.co < s.c_out ? m.co : s.c_out - 1;        // clamped: loads need no predicate
    const int n_q = (s.c_in + m.n_grp - 1) / m.n_grp;
    s.n_qp = (n_q + kAhead - 1) / kAhead * kAhead;
    return s;
}

// Request the weights of this lane's q-th input channel of a layer (all taps).  Past the end the
// last channel is fetched again: the loads stay unconditional.
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) v4f gfloat4;
__device__ __forceinline__ void fetch_w(float (&w)[kCasTapsPad], const WSrc &s, int q)
{
    int ci = s.grp + q * s.n_grp;
    ci = ci < s.c_in ? ci : s.c_in - 1;
    const gfloat4 *p = (const gfloat4 *)(s.w + (ci * s.c_out + s.co_c) * kCasTapsPad);
#pragma unroll
    for (int u = 0; u < kCasTapsPad / 4; ++u) {
        const v4f v = p[u];
        w[4 * u] = v.x; w[4 * u + 1] = v.y; w[4 * u + 2] = v.z; w[4 * u + 3] = v.w;
    }
}

// Step 2 for one layer.  wq holds the weights of this lane's first kAhead input channels; on
// return it holds those of the next layer's first kAhead channels.
template <int S, int NIN, int RHO>
__device__ __forceinline__ void accumulate(const float *__restrict__ x, int cnt, int co, int cp, const WSrc &cur,
                                           const WSrc &nxt, Wq &wq, float *__restrict__ red)
{
    constexpr int OFF = slot_off<S, RHO>();
    constexpr int TS = slot_cnt<S, NIN, RHO>();
    float acc[TS];
#pragma unroll
    for (int t = 0; t < TS; ++t) acc[t] = 0.f;
    const int n_q = (cur.c_in + cur.n_grp - 1) / cur.n_grp;  // input channels per lane, at most
    for (int qc = 0; qc < cur.n_qp; qc += kAhead) {
        float xv[kAhead][NIN];
#pragma unroll
        for (int p = 0; p < kAhead; ++p) {                    // all LDS reads of the batch first
            const int ci = cur.grp + (qc + p) * cur.n_grp;
            load_rows<NIN>(x + (ci < cur.c_in ? ci : cur.c_in - 1) * kXStride, xv[p]);
        }
#pragma unroll
        for (int p = 0; p < kAhead; ++p) {
            const int ci = cur.grp + (qc + p) * cur.n_grp;
            bool any = false;
#pragma unroll
            for (int j = 0; j < NIN; ++j) {
                if (j >= cnt) xv[p][j] = 0.f;                 // rows beyond the segment
                any |= xv[p][j] != 0.f;
            }
            if (qc + p < n_q && ci < cur.c_in && co < cur.c_out && any) {
#pragma unroll
                for (int j = 0; j < NIN; ++j) {
                    if (NIN <= 4 && xv[p][j] == 0.f) continue;            // zero: no event
#pragma unroll
                    for (int ky = 0; ky < kKMax; ++ky) {
                        if ((RHO + j - ky) % S != 0) continue;            // tap does not land on an output row
                        const int slot = (RHO + j - ky) / S - OFF;
                        acc[slot] = fmaf(xv[p][j], wq.w[p][ky], acc[slot]);
                    }
                }
            }
            // the slot is free: request what it will hold next, kAhead channels on -- which at
            // the end of this layer is the head of the next one
            const int qn = qc + p + kAhead;
            if (qn < cur.n_qp) fetch_w(wq.w[p], cur, qn);
            else fetch_w(wq.w[p], nxt, qn - cur.n_qp);
        }
    }
    if (co < cur.c_out) {
#pragma unroll
        for (int t = 0; t < TS; ++t) red[(cur.grp * kTMax + t) * cp + co] = acc[t];
    }
}

template <int S, int RHO>
__device__ __forceinline__ void accumulate_rows(const float *x, int cnt, int co, int cp, const WSrc &cur,
                                                const WSrc &nxt, Wq &wq, float *red)
{
    if (cnt <= 4) accumulate<S, 4, RHO>(x, cnt, co, cp, cur, nxt, wq, red);
    else accumulate<S, 16, RHO>(x, cnt, co, cp, cur, nxt, wq, red);
}

}  // namespace

int cascade1d_slot_off(int S, int rho) { return ceil_div_c(rho - kKMax + 1, S); }

__global__ void __launch_bounds__(kCasThreads) k_cascade1d(const CascadeArgs a_unused, const StreamSel sel)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    Lds &lds = *reinterpret_cast<Lds *>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int si = blockIdx.x;
    const int stream = sel_stream(sel, si);

    // The argument block (first kernel argument, offset 0 of the kernel-argument segment) goes to
    // LDS in one sweep: per-layer descriptors then cost an LDS read instead of a memory round trip.
    {
        const __attribute__((address_space(4))) uint32_t *kp =
            (const __attribute__((address_space(4))) uint32_t *)__builtin_amdgcn_kernarg_segment_ptr();
        for (int i = tid; i < kArgWords; i += kT) lds.args[i] = kp[i];
        if (tid < kCasMaxLayers) { lds.events[tid] = 0; lds.taps[tid] = 0; }
    }
    (void)a_unused;
    lds_barrier();
    const CascadeArgs &a = *reinterpret_cast<const CascadeArgs *>(lds.args);
    const int n_layers = a.n_layers;

    // Everything the chain needs from memory except the later weights, requested at once: the
    // first weights, the new input rows, the rolling buffers and biases of all layers.
    Wq wq;
    WSrc cur = wsrc_of(a, 0, tid);
#pragma unroll
    for (int p = 0; p < kAhead; ++p) fetch_w(wq.w[p], cur, p);
    {
        const int c0 = a.g[0].c_in, n = a.n_rows * c0;
        const gfloat *in = as_global((const float *)a.in) + (int64_t)(sel.pos0 + si) * a.in_stream_stride;
        unsigned int ev = 0, taps = 0;                          // the network input's events (eventise step)
        for (int i = tid; i < n; i += kT) {
            const int j = i / c0, c = i - j * c0;
            const float v = in[i];
            lds.x[0][c * kXStride + j] = v;
            if (v != 0.f) { ev += 1; taps += a.sched[0].taps[j]; }
        }
        if (a.stats && __ballot(ev != 0)) {
            for (int off = 32; off > 0; off >>= 1) { ev += __shfl_down(ev, off); taps += __shfl_down(taps, off); }
            if (lane == 0) { atomicAdd(&lds.events[0], ev); atomicAdd(&lds.taps[0], taps); }
        }
        for (int l = 0; l < n_layers; ++l) {
            const gfloat *ring = as_global((const float *)a.ring[l]) + (int64_t)stream * a.ring_stride[l];
            const int n_r = a.g[l].k_h * a.g[l].c_out;
            for (int i = tid; i < n_r; i += kT) lds.ring[l][i] = ring[i];
            const gfloat *bias = as_global((const float *)a.bias[l]);
            if (tid < a.g[l].c_out) lds.bias[l][tid] = bias ? bias[tid] : 0.f;
        }
    }
    lds_barrier();

    int cur_buf = 0;
    for (int l = 0; l < n_layers; ++l) {
        // this layer's step, copied out of LDS once (the barriers below would force re-reads)
        const CascadeLayer s = a.sched[l];
        const int cnt = s.cnt;
        if (cnt <= 0) break;
        const int c_out = cur.c_out, K = a.g[l].k_h, S = a.g[l].s_h, act = a.g[l].act;
        const float *x = lds.x[cur_buf];
        const bool more = l + 1 < n_layers && a.sched[l + 1].cnt > 0;
        const WSrc nxt = more ? wsrc_of(a, l + 1, tid) : cur;
        // per emitted row: the taps it lands on in layer l+1 (read by one lane per wave, from LDS)
        const unsigned char *taps_next = a.sched[more ? l + 1 : l].taps;

        // retained rows are read before anybody stores (a finished and a new row can share a slot)
        const Lanes m = lanes_of(s.cp_log, tid);
        float init[kCellsPerThread];
#pragma unroll
        for (int q = 0; q < kCellsPerThread; ++q) {
            const int idx = tid + q * kT;
            init[q] = 0.f;
            const int c = idx & (m.cp - 1), t = idx >> m.cp_log;
            if (t < s.t_lo || t >= s.t_hi || c >= c_out) continue;
            const bool fresh = s.d0 + t * S >= 0 || s.at_start;   // first input row of the row is new
            init[q] = fresh ? lds.bias[l][c] : lds.ring[l][((s.slot0 + t) % K) * c_out + c];
        }

        if (S == 1) accumulate_rows<1, 0>(x, cnt, m.co, m.cp, cur, nxt, wq, lds.red);
        else if (s.rho == 0) accumulate_rows<2, 0>(x, cnt, m.co, m.cp, cur, nxt, wq, lds.red);
        else accumulate_rows<2, 1>(x, cnt, m.co, m.cp, cur, nxt, wq, lds.red);
        lds_barrier();

        const bool last = l == n_layers - 1;
        gfloat *out = (gfloat *)a.out + (int64_t)stream * a.out_stride;
        const int64_t out_slot0 = a.out_slot0, out_cap = a.out_cap;
        const bool count = a.stats && more;
        float *xn = lds.x[cur_buf ^ 1];
        unsigned int ev = 0, taps = 0;
#pragma unroll
        for (int q = 0; q < kCellsPerThread; ++q) {
            const int idx = tid + q * kT;
            const int c = idx & (m.cp - 1), t = idx >> m.cp_log;
            const bool live = t >= s.t_lo && t < s.t_hi && c < c_out;
            bool emitted_nz = false;
            if (live) {
                float sum = init[q];
                const float *rp = lds.red + (t << m.cp_log) + c;
                const int g_stride = kTMax << m.cp_log;
                for (int gi = 0; gi < m.n_grp; gi += 8) {     // n_grp is a multiple of 8; fixed order
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = rp[(gi + u) * g_stride];
#pragma unroll
                    for (int u = 0; u < 8; ++u) sum += v[u];
                }
                if (t < s.t_fin) {
                    const float h = act == IDF_ACT_NONE ? sum : fmaxf(sum, 0.f);
                    if (last) {
                        int64_t slot = out_slot0 + (t - s.t_lo);
                        if (slot >= out_cap) slot -= out_cap;
                        out[slot * c_out + c] = h;
                    } else {
                        xn[c * kXStride + (t - s.t_lo)] = h;
                        emitted_nz = h != 0.f;
                    }
                } else {
                    lds.ring[l][((s.slot0 + t) % K) * c_out + c] = sum;
                }
            }
            // The non-zero values just emitted are the next layer's events: ballot them.  A wave
            // covers 64 / cp consecutive rows, cp lanes each.
            if (count) {
                const unsigned long long nzb = __ballot(emitted_nz);
                if (nzb && lane == 0) {
                    const int t0 = (tid + q * kT) >> m.cp_log;            // row of lane 0
                    const unsigned long long rowmask = m.cp == 64 ? ~0ull : ((1ull << m.cp) - 1ull);
                    for (int rr = 0; rr < (64 >> m.cp_log); ++rr) {
                        const int n = __popcll((nzb >> (rr << m.cp_log)) & rowmask);
                        const int j = t0 + rr - s.t_lo;
                        if (n && j >= 0 && j < kRowsMax) { ev += n; taps += n * taps_next[j]; }
                    }
                }
            }
        }
        if (count && lane == 0 && ev) { atomicAdd(&lds.events[l + 1], ev); atomicAdd(&lds.taps[l + 1], taps); }
        lds_barrier();
        cur_buf ^= 1;
        cur = nxt;
    }

    // the rolling buffers go back to memory, the counters are added up
    for (int l = 0; l < n_layers; ++l) {
        if (a.sched[l].cnt <= 0) break;
        gfloat *ring = (gfloat *)a.ring[l] + (int64_t)stream * a.ring_stride[l];
        const int n_r = a.g[l].k_h * a.g[l].c_out;
        for (int i = tid; i < n_r; i += kT) ring[i] = lds.ring[l][i];
    }
    if (a.stats && tid < n_layers && a.sched[tid].cnt > 0) {
        unsigned long long *dst = a.stats + ((int64_t)stream * n_layers + tid) * 2;
        if (lds.events[tid]) atomicAdd(dst, (unsigned long long)lds.events[tid]);
        if (lds.taps[tid]) atomicAdd(dst + 1, (unsigned long long)lds.taps[tid] * a.g[tid].c_out);
    }
}

bool cascade1d_eligible(int prec, const Geom *g, int n_layers, const int *rows_cap, int max_seg_rows)
{
    if (prec != IDF_PREC_F32 || n_layers > kCasMaxLayers || max_seg_rows > kCasRowsMax) return false;
    for (int l = 0; l < n_layers; ++l) {
        if (g[l].kind != IDF_CONV || g[l].w_in != 1 || g[l].w_out != 1 || g[l].k_w != 1) return false;
        if (g[l].c_in > 64 || g[l].c_out > 64 || g[l].k_h > kCasKMax || g[l].s_h > 2 || g[l].k_h < g[l].s_h) return false;
        if (g[l].act != IDF_ACT_NONE && g[l].act != IDF_ACT_RELU) return false;
        if (l < n_layers - 1 && rows_cap[l] > kCasRowsMax) return false;
    }
    return true;
}

hipError_t launch_cascade1d(const CascadeArgs &a, const StreamSel &sel, const LaunchCtx &lc)
{
    // more LDS than the default per-workgroup limit: raise it once
    static hipError_t prepared = hipFuncSetAttribute(reinterpret_cast<const void *>(k_cascade1d),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Lds));
    if (prepared != hipSuccess) return prepared;
    return launch(k_cascade1d, dim3(sel.n), dim3(kCasThreads), sizeof(Lds), lc, a, sel);
}

}  // namespace idf
