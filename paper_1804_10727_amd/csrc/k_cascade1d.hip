// Depth-first cascade for 1-D nets: one launch per push, one workgroup per stream, every
// layer the segment can influence handled in turn (Sec. 3 first paragraph: each segment goes
// through all of the network it can influence before the next is looked at).
//
// Per layer the workgroup
//   1. has the new input rows in LDS, stored per input channel ([channel][row]) so that one
//      wide LDS read brings all new rows of a channel;
//   2. accumulates w * dh (event-delivery rule of Sec. 3) with output channels across lanes
//      and the input channels dealt round-robin to groups of lanes.  A zero dh is not an
//      event and is branched over.  Each lane keeps the partial sums of all touched output
//      rows of its channel in registers -- the rolling buffer of K rows of Fig. 1 plus the
//      rows this segment completes; the register holding (input row j, tap ky) is fixed at
//      compile time, the weights of the next input channel are fetched while the current one
//      is being used;
//   3. adds the groups' partial sums in a fixed order to the retained pre-activations c (or
//      to the bias for rows touched for the first time), then either activates and emits the
//      row to the next layer (LDS) or stores it back as retained state.
//
// Serves float32 nets whose layers are all convolutions over a width-1 signal with at most 64
// channels, kernel height <= 9, stride <= 2 and at most 16 rows per layer per push.  Weights
// are expected zero-padded to 9 taps.
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

constexpr int ceil_div_c(int a, int b) { return a >= 0 ? (a + b - 1) / b : -((-a) / b); }
// Offset of accumulator slot 0 relative to floor((y0+p)/S), and number of slots.
template <int S, int RHO> constexpr int slot_off() { return ceil_div_c(RHO - kKMax + 1, S); }
template <int S, int NIN, int RHO> constexpr int slot_cnt() { return (RHO + NIN - 1) / S - slot_off<S, RHO>() + 1; }

struct Lds {
    float x[2][64 * kXStride];        // input rows of the current / next layer, [channel][row]
    float red[kT * kTMax];            // partial sums [group][slot][channel lane]
};

template <int NIN> __device__ __forceinline__ void load_rows(const float *p, float (&xv)[NIN])
{
    if constexpr (NIN >= 4) {
#pragma unroll
        for (int q = 0; q < NIN / 4; ++q) {
            const float4 v = *reinterpret_cast<const float4 *>(p + 4 * q);
            xv[4 * q] = v.x; xv[4 * q + 1] = v.y; xv[4 * q + 2] = v.z; xv[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < NIN; ++j) xv[j] = p[j];
    }
}

// Step 2 for one layer.
template <int S, int NIN, int RHO>
__device__ __forceinline__ void accumulate(const float *__restrict__ x, const float *__restrict__ w, int cnt,
                                           int c_in, int c_out, int cp, int co, int grp, int n_grp,
                                           float *__restrict__ red)
{
    constexpr int OFF = slot_off<S, RHO>();
    constexpr int TS = slot_cnt<S, NIN, RHO>();
    if (co >= c_out) return;
    float acc[TS];
#pragma unroll
    for (int t = 0; t < TS; ++t) acc[t] = 0.f;
    const int tap_stride = c_in * c_out;
    float wk[kKMax];
    int ci = grp;
    if (ci < c_in) {
#pragma unroll
        for (int ky = 0; ky < kKMax; ++ky) wk[ky] = w[ky * tap_stride + ci * c_out + co];
    }
    for (; ci < c_in; ci += n_grp) {
        float wn[kKMax];
        const int cn = ci + n_grp;
#pragma unroll
        for (int ky = 0; ky < kKMax; ++ky) wn[ky] = cn < c_in ? w[ky * tap_stride + cn * c_out + co] : 0.f;
        float xv[NIN];
        load_rows<NIN>(x + ci * kXStride, xv);
#pragma unroll
        for (int j = 0; j < NIN; ++j) {
            if (j >= cnt || xv[j] == 0.f) continue;          // zero: no event
#pragma unroll
            for (int ky = 0; ky < kKMax; ++ky) {
                if ((RHO + j - ky) % S != 0) continue;        // tap does not land on an output row
                const int slot = (RHO + j - ky) / S - OFF;
                acc[slot] = fmaf(xv[j], wk[ky], acc[slot]);
            }
        }
#pragma unroll
        for (int ky = 0; ky < kKMax; ++ky) wk[ky] = wn[ky];
    }
#pragma unroll
    for (int t = 0; t < TS; ++t) red[(grp * kTMax + t) * cp + co] = acc[t];
}

template <int S, int RHO>
__device__ __forceinline__ void accumulate_rows(const float *x, const float *w, int cnt, int c_in, int c_out, int cp,
                                                int co, int grp, int n_grp, float *red)
{
    if (cnt <= 1) accumulate<S, 1, RHO>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, red);
    else if (cnt <= 2) accumulate<S, 2, RHO>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, red);
    else if (cnt <= 4) accumulate<S, 4, RHO>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, red);
    else if (cnt <= 8) accumulate<S, 8, RHO>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, red);
    else accumulate<S, 16, RHO>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, red);
}

}  // namespace

int cascade1d_slot_off(int S, int rho) { return ceil_div_c(rho - kKMax + 1, S); }

__global__ void __launch_bounds__(kCasThreads) k_cascade1d(const CascadeArgs a, const StreamSel sel)
{
    __shared__ __attribute__((aligned(16))) Lds lds;
    const int tid = threadIdx.x;
    const int si = blockIdx.x;
    const int stream = sel_stream(sel, si);

    // network input rows -> LDS, transposed to [channel][row]
    int cur = 0;
    {
        const int c0 = a.g[0].c_in, n = a.n_rows * c0;
        const float *in = (const float *)a.in + (int64_t)(sel.pos0 + si) * a.in_stream_stride;
        for (int i = tid; i < n; i += kT) {
            const int j = i / c0, c = i - j * c0;
            lds.x[0][c * kXStride + j] = in[i];
        }
    }
    __syncthreads();

    for (int l = 0; l < a.n_layers; ++l) {
        const CascadeLayer &s = a.sched[l];
        const int cnt = s.cnt;
        if (cnt <= 0) break;
        const Geom &g = a.g[l];
        const int c_in = g.c_in, c_out = g.c_out, K = g.k_h, S = g.s_h;
        const float *x = lds.x[cur];

        // counters: events delivered to this layer and the multiply-adds they stand for
        if (tid < 64 && a.stats) {
            unsigned int ev = 0, taps = 0;
            if (tid < cnt) {
                for (int ci = 0; ci < c_in; ++ci) ev += x[ci * kXStride + tid] != 0.f ? 1u : 0u;
                taps = ev * s.taps[tid];
            }
            for (int off = 32; off > 0; off >>= 1) { ev += __shfl_down(ev, off); taps += __shfl_down(taps, off); }
            if (tid == 0) {
                unsigned long long *dst = a.stats + ((int64_t)stream * a.n_layers + l) * 2;
                if (ev) atomicAdd(dst, (unsigned long long)ev);
                if (taps) atomicAdd(dst + 1, (unsigned long long)taps * c_out);
            }
        }

        // lanes: channel within the power-of-two pad of c_out; groups share the input channels
        const int cp_log = s.cp_log, cp = 1 << cp_log;
        const int co = tid & (cp - 1), grp = tid >> cp_log, n_grp = kT >> cp_log;

        // retained rows are fetched before anybody stores (a finished and a new row can share a
        // ring slot); the loads stay in flight during the accumulation
        float *ring = (float *)a.ring[l] + (int64_t)stream * a.ring_stride[l];
        const float *bias = (const float *)a.bias[l];
        float init[kCellsPerThread];
#pragma unroll
        for (int q = 0; q < kCellsPerThread; ++q) {
            const int idx = tid + q * kT;
            init[q] = 0.f;
            const int c = idx & (cp - 1), t = idx >> cp_log;
            if (t < s.t_lo || t >= s.t_hi || c >= c_out) continue;
            const bool fresh = s.d0 + t * S >= 0 || s.at_start;   // first input row of the row is new
            init[q] = fresh ? (bias ? bias[c] : 0.f) : ring[((s.slot0 + t) % K) * c_out + c];
        }

        const float *w = (const float *)a.w[l];
        if (S == 1) accumulate_rows<1, 0>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, lds.red);
        else if (s.rho == 0) accumulate_rows<2, 0>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, lds.red);
        else accumulate_rows<2, 1>(x, w, cnt, c_in, c_out, cp, co, grp, n_grp, lds.red);
        __syncthreads();

        const bool last = l == a.n_layers - 1;
        float *xn = lds.x[cur ^ 1];
#pragma unroll
        for (int q = 0; q < kCellsPerThread; ++q) {
            const int idx = tid + q * kT;
            const int c = idx & (cp - 1), t = idx >> cp_log;
            if (t < s.t_lo || t >= s.t_hi || c >= c_out) continue;
            float sum = init[q];
            for (int gi = 0; gi < n_grp; ++gi) sum += lds.red[((gi * kTMax + t) << cp_log) + c];
            if (t < s.t_fin) {
                const float h = g.act == IDF_ACT_NONE ? sum : fmaxf(sum, 0.f);
                if (last) {
                    int64_t slot = a.out_slot0 + (t - s.t_lo);
                    if (slot >= a.out_cap) slot -= a.out_cap;
                    ((float *)a.out)[(int64_t)stream * a.out_stride + slot * c_out + c] = h;
                } else {
                    xn[c * kXStride + (t - s.t_lo)] = h;
                }
            } else {
                ring[((s.slot0 + t) % K) * c_out + c] = sum;
            }
        }
        __syncthreads();
        cur ^= 1;
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
    return launch(k_cascade1d, dim3(sel.n), dim3(kCasThreads), 0, lc, a, sel);
}

}  // namespace idf
