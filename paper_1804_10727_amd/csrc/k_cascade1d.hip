// Depth-first cascade for 1-D nets: one launch per push, one workgroup per stream and stage,
// every layer the segment can influence handled in turn (Sec. 3 first paragraph: each segment
// goes through all of the network it can influence before the next is looked at).
//
// The stream's whole retained state -- the rolling buffer of K rows of pre-activations c of
// every layer (Fig. 1) -- is brought into LDS when the kernel starts, lives there while the
// segment runs through the layers; rows that stay unfinished go back to memory as they are
// summed.  Per layer the workgroup
//   1. has the new input rows in LDS, stored per input channel ([channel][row], rows past the
//      segment zero) so that one wide LDS read brings all new rows of a channel, next to a bit
//      per channel telling whether any of them holds an event;
//   2. accumulates w * dh (event-delivery rule of Sec. 3) with output channels across lanes
//      and the input channels dealt round-robin to groups of lanes.  Zero values are not
//      events: a channel without an event in the segment is skipped.  Each lane keeps the
//      partial sums of all touched output rows of its channel in registers; the register
//      holding (input row j, tap ky) is fixed at compile time;
//   3. adds the groups' partial sums in a fixed order to the retained c (or to the bias for
//      rows touched for the first time), then either activates and emits the row to the next
//      layer (LDS) -- a wave ballot of the non-zero values it emits gives the next layer's
//      events and channel bits -- or keeps it for the rolling buffer.
//
// A workgroup is a chain of dependent layers run by four waves (two workgroups share a compute
// unit, so that the waiting of one runs under the arithmetic of the other), and what limits it
// is the number of instructions a wave has to issue (one per four cycles):
// hence per channel a handful of instructions besides the multiply-adds themselves -- running
// offsets instead of address arithmetic, no per-row masks, one bit test for silence -- and
// variants for 4, 8 and 16 new rows.  Every weight is needed exactly once per push; the
// weights are one continuous stream of requests running four input channels ahead of their
// use, across layer boundaries (the tail of layer l already requests the head of layer l+1).
//
// Serves float32 nets whose layers are all convolutions over a width-1 signal with at most 64
// channels, kernel height <= 9, stride <= 2 and at most 16 rows per layer per push.  Weights
// come in a packing of their own (cascade1d_weight_index): two 16-byte loads and one 4-byte
// load per channel pair, each wave-wide load covering whole cache lines, input channels
// padded with zeros so that every lane can run the same number of steps.
#include <cstring>

#include "idf.h"
#include "idf_kernels.h"
#include <cstddef>

namespace idf {

namespace {

constexpr int kT = kCasThreads;
constexpr int kKMax = kCasKMax;
constexpr int kTMax = kCasSlotsMax;                  // touched output rows at most
constexpr int kCellsPerThread = (kTMax * 64 + kT - 1) / kT;
constexpr int kXStride = 20;                         // floats per channel in LDS (16 rows + pad, 16-byte aligned)
constexpr int kAhead = kCasAhead;                    // input channels whose weights are in flight
constexpr int kBatch = 4;                            // input channels whose rows are read from LDS together
constexpr int kArgWords = (sizeof(CascadeArgs) + 3) / 4;
static_assert(offsetof(CascadeArgs, step) % 4 == 0 && (sizeof(CascadeStep) * kCasMaxLayers) % 4 == 0, "copied word by word");
static_assert(offsetof(CascadeArgsT<1>, step) == offsetof(CascadeArgs, step) && offsetof(CascadeArgsT<1>, in) == offsetof(CascadeArgs, in) &&
              offsetof(CascadeArgsT<1>, in_stream_stride) == offsetof(CascadeArgs, in_stream_stride), "the short block is a prefix of the long one");
constexpr int kRingPerLayer = kKMax * 64;            // floats of rolling buffer per layer at most
constexpr int kXinPerLane = (kCasRowsMax * 64 + kT - 1) / kT;      // values of a segment per lane at most
constexpr int kRingPerLane = (kRingPerLayer + kT - 1) / kT;
constexpr int kRedU = kT / 64 < 8 ? kT / 64 : 8;     // partial sums gathered per round: divides every number of lane groups

constexpr int ceil_div_c(int a, int b) { return a >= 0 ? (a + b - 1) / b : -((-a) / b); }
// Offset of accumulator slot 0 relative to floor((y0+p)/S), and number of slots.
template <int S, int RHO> constexpr int slot_off() { return ceil_div_c(RHO - kKMax + 1, S); }
template <int S, int NIN, int RHO> constexpr int slot_cnt() { return (RHO + NIN - 1) / S - slot_off<S, RHO>() + 1; }

struct Lds {
    float x[2][64 * kXStride];                   // input rows of the current / next layer, [channel][row]
    float red[kT * kTMax];                       // partial sums [group][slot][channel lane]
    float ring[kCasMaxLayers][kRingPerLayer];    // the stream's rolling buffers, [layer][slot][channel]
    float bias[kCasMaxLayers][64];
    unsigned int chmask[2][2];                   // per x buffer: bit c set when channel c holds an event
    unsigned long long nzlog[kCasMaxLayers][kT / 64][kCellsPerThread];   // ballots of emitted non-zeros
    uint32_t args[kArgWords];                    // the kernel's argument block
};

// Pointers read back from LDS have lost their address space; saying "global" again lets the
// compiler use global (not flat) loads, whose completion order it can count on.
typedef __attribute__((address_space(1))) float gfloat;
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) v4f gfloat4;
template <class P> __device__ __forceinline__ const gfloat *as_global(const P *p) { return (const gfloat *)p; }
// The same for a pointer every lane holds alike: kept in scalar registers, so that a load is
// "scalar base + per-lane offset" with no 64-bit arithmetic per lane.
__device__ __forceinline__ const gfloat *uniform_global(const void *p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const gfloat *)(((uint64_t)hi << 32) | lo);
}

struct Wq { float w[kAhead][kKMax]; };           // weights of kAhead input channels, all taps

// A lane's place in the weight stream of one layer: byte offsets of its next input channel in
// the two 4-tap groups and in the ninth-tap plane, and the steps to the channel after.
struct WCur {
    const __attribute__((address_space(1))) char *w;
    uint32_t o4, o4b, o8, step4, step8;
};

// Lane mapping of one layer: channel lane within the power-of-two pad of c_out, group of lanes.
struct Lanes { int cp_log, cp, co, grp, n_grp; };
__device__ __forceinline__ Lanes lanes_of(int cp_log, int tid)
{
    Lanes m;
    m.cp_log = cp_log; m.cp = 1 << cp_log;
    m.co = tid & (m.cp - 1); m.grp = tid >> cp_log; m.n_grp = kT >> cp_log;
    return m;
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }   // same in every lane: keep it scalar

// The cursor at the lane's first input channel of a layer.
__device__ __forceinline__ WCur cursor_of(const CascadeLayer &sl, int tid)
{
    const int cp_log = uni(sl.cp_log), c_out = uni(sl.c_out), n_qp = uni(sl.steps);
    const Lanes m = lanes_of(cp_log, tid);
    WCur s;
    s.w = (const __attribute__((address_space(1))) char *)uniform_global(sl.w);
    const int co_c = m.co < c_out ? m.co : c_out - 1;        // clamped: loads need no predicate
    s.o4 = (uint32_t)((m.grp * 2 * c_out + co_c) * 16);
    s.o4b = s.o4 + (uint32_t)(c_out * 16);
    s.o8 = (uint32_t)(((m.n_grp * n_qp * 8 + m.grp) * c_out + co_c) * 4);
    s.step4 = (uint32_t)(m.n_grp * 2 * c_out * 16);
    s.step8 = (uint32_t)(m.n_grp * c_out * 4);
    return s;
}

// Request the weights (all taps) of the input channel the cursor stands on, and move it on.  A
// cursor may run over its layer's steps (a multiple of kAhead), and over the first kAhead
// channels of any layer: the packing is padded to that.
static_assert(kKMax == 9, "the weight packing is two 16-byte groups and one single tap");
__device__ __forceinline__ void fetch_w(float (&w)[kKMax], WCur &s)
{
    const v4f a = *(const gfloat4 *)(s.w + s.o4);
    const v4f b = *(const gfloat4 *)(s.w + s.o4b);
    w[8] = *(const gfloat *)(s.w + s.o8);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w;
    w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
    s.o4 += s.step4; s.o4b += s.step4; s.o8 += s.step8;
}

template <int NIN> __device__ __forceinline__ void load_rows(const float *p, float (&xv)[NIN])
{
#pragma unroll
    for (int q = 0; q < NIN / 4; ++q) {
        const float4 v = *reinterpret_cast<const float4 *>(p + 4 * q);
        xv[4 * q] = v.x; xv[4 * q + 1] = v.y; xv[4 * q + 2] = v.z; xv[4 * q + 3] = v.w;
    }
}

// Step 2 for one layer of n_qp steps.  wq holds the weights of this lane's first kAhead input
// channels and wc stands on the channel after them; on return the same holds for the next
// layer, whose cursor at its first channel is nxt0.  visit: this lane's view
// of the channel bits, already shifted so that bit 0 belongs to its first channel (all zero
// for lanes beyond c_out).
template <int S, int NIN, int RHO>
__device__ __forceinline__ void accumulate(const float *__restrict__ x, const Lanes &m, int n_qp, WCur &wc, const WCur &nxt0,
                                           Wq &wq, unsigned long long visit, float *__restrict__ red)
{
    constexpr int OFF = slot_off<S, RHO>();
    constexpr int TS = slot_cnt<S, NIN, RHO>();
    float acc[TS];
#pragma unroll
    for (int t = 0; t < TS; ++t) acc[t] = 0.f;
    // moving on by n_grp channels: two shifts of at most 32 (a single shift by 64 or more is not defined)
    const int sh1 = m.n_grp < 32 ? m.n_grp : 32, sh2 = m.n_grp - sh1 < 32 ? m.n_grp - sh1 : 32;
    int ci = m.grp;
    for (int qc = 0; qc < n_qp; qc += kAhead) {
        if (qc + kAhead >= n_qp) wc = nxt0;                       // the tail of this layer requests the head of the next
#pragma unroll
        for (int h = 0; h < kAhead; h += kBatch) {
            float xv[kBatch][NIN];
#pragma unroll
            for (int p = 0; p < kBatch; ++p) {                // all LDS reads of the batch first
                const int cc = ci + p * m.n_grp;
                load_rows<NIN>(x + (cc < 63 ? cc : 63) * kXStride, xv[p]);
            }
#pragma unroll
            for (int p = 0; p < kBatch; ++p) {
                if (visit & 1ull) {
#pragma unroll
                    for (int j = 0; j < NIN; ++j) {
#pragma unroll
                        for (int ky = 0; ky < kKMax; ++ky) {
                            if ((RHO + j - ky) % S != 0) continue;        // tap does not land on an output row
                            const int slot = (RHO + j - ky) / S - OFF;
                            acc[slot] = fmaf(xv[p][j], wq.w[h + p][ky], acc[slot]);
                        }
                    }
                }
                visit = (visit >> sh1) >> sh2;
                fetch_w(wq.w[h + p], wc);     // the slot is free: request what it will hold next, kAhead channels on
            }
            ci += kBatch * m.n_grp;
        }
    }
    float *rp = red + ((m.grp * kTMax) << m.cp_log) + m.co;
#pragma unroll
    for (int t = 0; t < TS; ++t) rp[t << m.cp_log] = acc[t];
}

template <int S, int RHO>
__device__ __forceinline__ void accumulate_rows(const float *x, int cnt, const Lanes &m, int n_qp, WCur &wc, const WCur &nxt0,
                                                Wq &wq, unsigned long long visit, float *red)
{
    if (cnt <= 4) accumulate<S, 4, RHO>(x, m, n_qp, wc, nxt0, wq, visit, red);
    else if (cnt <= 8) accumulate<S, 8, RHO>(x, m, n_qp, wc, nxt0, wq, visit, red);
    else accumulate<S, 16, RHO>(x, m, n_qp, wc, nxt0, wq, visit, red);
}

// OR of the cp-bit fields of a 64-bit ballot (cp a power of two): which channels had a hit.
__device__ __forceinline__ unsigned long long fold_channels(unsigned long long b, int cp)
{
    for (int w = 32; w >= cp; w >>= 1) b |= b >> w;
    return cp == 64 ? b : b & ((1ull << cp) - 1ull);
}

}  // namespace

// Weight packing: taps 0..7 as [c_in][2][c_out][4] (a wave's 16-byte loads tile whole cache
// lines), then tap 8 as [c_in][c_out]; c_in counted with its zero padding
// (cascade1d_cin_pad), kernels shorter than 9 taps zero padded.
size_t cascade1d_weight_index(int c_in, int c_out, int ci, int co, int ky)
{
    if (ky < 8) return (((size_t)ci * 2 + ky / 4) * c_out + co) * 4 + ky % 4;
    return ((size_t)cascade1d_cin_pad(c_in, c_out) * 8 + ci) * c_out + co;
}

int cascade1d_slot_off(int S, int rho) { return ceil_div_c(rho - kKMax + 1, S); }

template <bool COUNT, int NSTEP>
__global__ void __launch_bounds__(kCasThreads, 2) k_cascade1d(const CascadeArgsT<NSTEP> ka, const StreamSel sel)
{
    constexpr int kArgWords = (sizeof(CascadeArgsT<NSTEP>) + 3) / 4;         // this launch's block: the short one when every stage runs one step
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    Lds &lds = *reinterpret_cast<Lds *>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63;
    // The grid is (streams side by side, stage, groups of streams).  Workgroups go to the eight XCDs
    // in turn by their linear number; with `per` = 8 / stages streams side by side, stage s meets XCDs
    // s*per .. s*per+per-1 only, so its weights are fetched into the L2 of its XCDs, not into all eight.
    // The stage comes from the grid index and the stage's first layer from a copy indexed by stage:
    // everything the first memory requests need is then one round of scalar loads away (looked up
    // through the stage table it was three dependent rounds, about a microsecond per launch).
    const int stage = blockIdx.y;
    // The argument block (first kernel argument, offset 0 of the kernel-argument segment) goes to
    // LDS in one sweep: inside the chain a layer's descriptor then costs an LDS read instead of a
    // memory round trip.  The prologue itself reads the arguments as scalars, so that everything
    // the chain needs from memory except the later weights is requested at once, next to that
    // sweep: the first weights, the new input rows, the rolling buffers and biases of the firing
    // layers.
    // (Requested before anything else: its latency then runs under the scalar loads below.)
    constexpr int kArgPerLane = (kArgWords + kT - 1) / kT;
    uint32_t argw[kArgPerLane];
    {
        const __attribute__((address_space(4))) uint32_t *kp =
            (const __attribute__((address_space(4))) uint32_t *)__builtin_amdgcn_kernarg_segment_ptr();
#pragma unroll
        for (int u = 0; u < kArgPerLane; ++u) {
            const int i = tid + u * kT;
            argw[u] = kp[i < kArgWords ? i : kArgWords - 1];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    const int si = blockIdx.z * ka.per + blockIdx.x;
    const int stream = sel_stream(sel, si);
    const int n_layers = ka.n_layers;
    const int lb = ka.stage_lo[stage], le = ka.stage_lo[stage + 1];
    const int n_seg = ka.stage_steps[stage];                     // steps this stage runs one after the other
    const CascadeLayer &first = ka.first[stage];
    const CascadeStep &first_step = ka.first_step[stage];
    // First round of scalar loads, asked for in one batch with one wait (left to first use they
    // end up behind conditions, one memory round trip each, one after the other).
    asm volatile("" ::"s"(ka.per), "s"(sel.n), "s"(sel.base), "s"(sel.pos0), "s"(n_layers), "s"(lb), "s"(le), "s"(n_seg),
                 "s"((int)first_step.cnt), "s"(first.c_in), "s"(first.c_out), "s"(first.cp_log), "s"(first.steps), "s"(first.w),
                 "s"(ka.in[0]), "s"(ka.in_stream_stride[0]), "s"(ka.transit), "s"(ka.transit_stream_stride),
                 "s"(ka.transit_buf_stride), "s"(ka.transit_wr), "s"(ka.stats));
    if (n_seg <= 0) return;                                      // nothing has reached this stage
    Wq wq;
    WCur wc = cursor_of(first, tid);
#pragma unroll
    for (int p = 0; p < kAhead; ++p) fetch_w(wq.w[p], wc);
    const int c0 = first.c_in;
    // The new rows of segment q for this stage's first layer: the pushed segment, or the rows the
    // stage before handed over in the previous launch.  Asked for one segment ahead of their use.
    const gfloat *tr_in = as_global((const float *)ka.transit) + ((stage - 1) * 2 + (ka.transit_wr ^ 1)) * ka.transit_buf_stride +
                          (int64_t)stream * ka.transit_stream_stride;
    float xin[kXinPerLane];
    // A step of stage 0 takes the rows of one pushed segment or gathers those of several; the table of
    // segments is read as scalars for the launch's first step when that is one segment (the usual
    // launch per push: nothing may wait for the copy of the arguments on chip), from that copy later.
    const __attribute__((address_space(4))) char *kargs = (const __attribute__((address_space(4))) char *)__builtin_amdgcn_kernarg_segment_ptr();
    auto request_rows = [&](const CascadeStep &st, const CascadeArgs *on_chip) {
        const int n_in = st.cnt * c0;                            // at most 16 rows x 64 channels
        if (stage == 0 && !on_chip && st.cnt <= st.seg_rows) {
            const gfloat *in = as_global((const float *)ka.in[0]) + (int64_t)(sel.pos0 + si) * ka.in_stream_stride[0];
#pragma unroll
            for (int u = 0; u < kXinPerLane; ++u) {
                const int i = tid + u * kT;
                xin[u] = in[n_in > 0 ? (i < n_in ? i : n_in - 1) : 0];
            }
        } else if (stage == 0) {
            const int per_seg = st.seg_rows * c0;                // values one pushed segment brings (at most 16 x 64)
            // i / per_seg through a float: (i + 0.5) / per_seg is at least 0.5 / 1024 away from every integer,
            // the rounding of the product stays far below that
            const float inv = 1.0f / (float)(per_seg > 0 ? per_seg : 1);
#pragma unroll
            for (int u = 0; u < kXinPerLane; ++u) {
                int i = tid + u * kT;
                i = n_in > 0 ? (i < n_in ? i : n_in - 1) : 0;
                const int sq = (int)(((float)i + 0.5f) * inv), within = i - sq * per_seg;
                const int q = st.seg0 + (n_in > 0 ? sq : 0);
                uint64_t base;
                int stride;
                if (on_chip) {
                    base = (uint64_t)on_chip->in[q]; stride = on_chip->in_stream_stride[q];
                } else {
                    base = *(const __attribute__((address_space(4))) uint64_t *)(kargs + offsetof(CascadeArgs, in) + q * 8);
                    stride = *(const __attribute__((address_space(4))) int *)(kargs + offsetof(CascadeArgs, in_stream_stride) + q * 4);
                }
                xin[u] = ((const gfloat *)base)[(int64_t)(sel.pos0 + si) * stride + within];
            }
        } else {
            const gfloat *in = tr_in + st.in_off * c0;
#pragma unroll
            for (int u = 0; u < kXinPerLane; ++u) {
                const int i = tid + u * kT;
                xin[u] = in[n_in > 0 ? (i < n_in ? i : n_in - 1) : 0];
            }
        }
    };
    request_rows(first_step, nullptr);
    // Second round: what the rolling-buffer requests of the stage's layers need.  The first
    // kPinned layers of the stage in one batch; a stage with more layers (a deep net run without
    // stages) fetches the rest as it goes.
    constexpr int kPinned = 3;
    const int l_last = n_layers - 1;
    auto layer_of = [&](int j) -> const CascadeLayer & { return ka.layer[lb + j < l_last ? lb + j : l_last]; };
    {
        const CascadeLayer &q0 = layer_of(0), &q1 = layer_of(1), &q2 = layer_of(2);
        static_assert(kPinned == 3, "one group of operands per pinned layer");
        asm volatile("" ::"s"(q0.ring), "s"(q0.ring_stride), "s"(q0.ring_floats), "s"(q0.bias), "s"(q0.c_out),
                     "s"(q1.ring), "s"(q1.ring_stride), "s"(q1.ring_floats), "s"(q1.bias), "s"(q1.c_out),
                     "s"(q2.ring), "s"(q2.ring_stride), "s"(q2.ring_floats), "s"(q2.bias), "s"(q2.c_out));
    }

    // The rolling buffers of the stage's layers come into LDS once and stay there while the
    // launch's segments run through (rows left unfinished are written to LDS and to memory alike).
    float rv[kCasMaxLayers][kRingPerLane], bv[kCasMaxLayers];             // by position in the stage: layer lb + j
#pragma unroll
    for (int j = 0; j < kCasMaxLayers; ++j) {
        bv[j] = 0.f;
#pragma unroll
        for (int u = 0; u < kRingPerLane; ++u) rv[j][u] = 0.f;
        const CascadeLayer &sl = layer_of(j);
        if (lb + j < le) {
            const gfloat *ring = as_global((const float *)sl.ring) + (int64_t)stream * sl.ring_stride;
            const int n_r = sl.ring_floats;
#pragma unroll
            for (int u = 0; u < kRingPerLane; ++u) {
                const int i = tid + u * kT;
                rv[j][u] = ring[i < n_r ? i : n_r - 1];
            }
            const gfloat *bias = as_global((const float *)sl.bias);
            if (bias) bv[j] = bias[tid < sl.c_out ? tid : sl.c_out - 1];
        }
    }
    {
        if (tid < 4) lds.chmask[tid >> 1][tid & 1] = 0;
        for (int i = tid; i < 64 * kXStride / 4; i += kT)       // rows past the segment read as zero
            reinterpret_cast<float4 *>(lds.x[0])[i] = float4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < kArgPerLane; ++u) {
            const int i = tid + u * kT;
            if (i < kArgWords) lds.args[i] = argw[u];
        }
#pragma unroll
        for (int j = 0; j < kCasMaxLayers; ++j) {
            if (lb + j < le) {
#pragma unroll
                for (int u = 0; u < kRingPerLane; ++u)
                    if (tid + u * kT < kRingPerLayer) lds.ring[lb + j][tid + u * kT] = rv[j][u];
                if (tid < 64) lds.bias[lb + j][tid] = bv[j];
            }
        }
    }
    lds_barrier();
    const CascadeArgs &a = *reinterpret_cast<const CascadeArgs *>(lds.args);

    for (int seg = 0; seg < n_seg; ++seg) {
    const int cnt0 = uni(a.step[seg][lb].cnt);
    // (x[0] and its channel bits are clear here: by the prologue, or by the end of the segment before)
    if (cnt0 > 0) {
        const int n_in = cnt0 * c0;
        unsigned int ev = 0, taps = 0;                          // the network input's events (eventise step)
#pragma unroll
        for (int u = 0; u < kXinPerLane; ++u) {
            const int i = tid + u * kT;
            if (i < n_in && xin[u] != 0.f) {
                const int j = i / c0, c = i - j * c0;
                lds.x[0][c * kXStride + j] = xin[u];
                atomicOr(&lds.chmask[0][c >> 5], 1u << (c & 31));
                ev += 1; taps += cascade_taps(a.step[seg][lb], j);
            }
        }
        if (ka.stats && __ballot(ev != 0)) {
            for (int off = 32; off > 0; off >>= 1) { ev += __shfl_down(ev, off); taps += __shfl_down(taps, off); }
            if (lane == 0) {
                unsigned long long *dst = ka.stats + ((int64_t)stream * n_layers + lb) * 2;
                atomicAdd(dst, (unsigned long long)ev);
                atomicAdd(dst + 1, (unsigned long long)taps * first.c_out);
            }
        }
    }
    if (seg + 1 < n_seg) request_rows(a.step[seg + 1][lb], &a);  // the next step's rows, on their way while this one runs
    lds_barrier();

    int cur_buf = 0;
    for (int l = lb; l < le; ++l) {
        // this layer's step: scalars copied out of LDS once (the barriers below would force re-reads)
        const CascadeLayer &sl = a.layer[l];
        const CascadeStep &ss = a.step[seg][l];
        const int cnt = uni(ss.cnt);
        if (cnt <= 0) break;
        const int t_lo = uni(ss.t_lo), t_fin = uni(ss.t_fin), t_hi = uni(ss.t_hi), d0 = uni(ss.d0);
        const int at_start = uni(ss.at_start), rho = uni(ss.rho), cp_log = uni(sl.cp_log);
        const int c_out = uni(sl.c_out), c_in = uni(sl.c_in), S = uni(sl.s_h), act = uni(sl.act);
        const int K = uni(sl.k_h), slot0 = uni(ss.slot0), rcp_k = uni(sl.rcp_k);
        gfloat *ringg = (gfloat *)uniform_global(sl.ring) + (int64_t)stream * sl.ring_stride;
        const float *x = lds.x[cur_buf];
        float *xn = lds.x[cur_buf ^ 1];
        const bool more = l + 1 < le && uni(a.step[seg][l + 1].cnt) > 0;
        // whose weights the tail of this layer asks for: the next layer's, or, when the segment ends
        // here and another follows, those of the stage's first layer again
        const WCur nxt0 = cursor_of(a.layer[more ? l + 1 : (seg + 1 < n_seg ? lb : l)], tid);
        const int n_qp = uni(sl.steps);
        // groups of lanes beyond the input channels hold no partial sums (they write zeros): not read
        const int n_red = (kT >> cp_log) < ((c_in + kRedU - 1) & ~(kRedU - 1)) ? (kT >> cp_log) : ((c_in + kRedU - 1) & ~(kRedU - 1));
        const Lanes m = lanes_of(cp_log, tid);

        // this lane's view of the channel bits: bit q*n_grp of it belongs to its q-th channel
        unsigned long long visit = ((unsigned long long)lds.chmask[cur_buf][1] << 32) | lds.chmask[cur_buf][0];
        visit = (m.grp < 64 && m.co < c_out) ? visit >> m.grp : 0ull;
        // the other buffer is free (its readers are past the previous layer's first barrier):
        // clear it for the rows this layer emits
        for (int i = tid; i < 64 * kXStride / 4; i += kT) reinterpret_cast<float4 *>(xn)[i] = float4{0.f, 0.f, 0.f, 0.f};
        if (COUNT && ka.issued && tid == 0) {
            const int n_ev = __popc(lds.chmask[cur_buf][0]) + __popc(lds.chmask[cur_buf][1]);
            if (n_ev) atomicAdd(ka.issued + (int64_t)stream * n_layers + l, (unsigned long long)n_ev * uni(ss.fma_per_channel) * c_out);
        }
        if (tid < 2) lds.chmask[cur_buf ^ 1][tid] = 0;

        if (S == 1) accumulate_rows<1, 0>(x, cnt, m, n_qp, wc, nxt0, wq, visit, lds.red);
        else if (rho == 0) accumulate_rows<2, 0>(x, cnt, m, n_qp, wc, nxt0, wq, visit, lds.red);
        else accumulate_rows<2, 1>(x, cnt, m, n_qp, wc, nxt0, wq, visit, lds.red);
        lds_barrier();

        // Step 3.  Every lane owns up to kCellsPerThread (row, channel) cells; all LDS reads of
        // all its cells are issued before anything is summed.
        const bool last = l == n_layers - 1, hand_over = l == le - 1 && !last;
        gfloat *tr = (gfloat *)ka.transit + (stage * 2 + ka.transit_wr) * ka.transit_buf_stride +
                     (int64_t)stream * ka.transit_stream_stride + uni(ss.out_off) * c_out;
        const int rows_per_pass = kT >> cp_log;
        const int c = tid & (m.cp - 1), cc = c < c_out ? c : c_out - 1;
        int t_of[kCellsPerThread], at[kCellsPerThread];
        bool live[kCellsPerThread];
        float sum[kCellsPerThread], ringv[kCellsPerThread];
        const float bias_c = lds.bias[l][cc];
#pragma unroll
        for (int q = 0; q < kCellsPerThread; ++q) {
            const int t = t_lo + (tid >> cp_log) + q * rows_per_pass;
            live[q] = t < t_hi && c < c_out;
            t_of[q] = t < t_hi ? t : (t_hi > t_lo ? t_hi - 1 : t_lo);   // clamped: reads need no predicate
            const int v = slot0 + t_of[q];
            at[q] = (v - ((v * rcp_k) >> 16) * K) * c_out + cc;   // ring slot (slot0 + t) mod K
            ringv[q] = lds.ring[l][at[q]];
        }
        {
            const int g_stride = kTMax << cp_log;
            bool wave_has[kCellsPerThread];                   // some lane of this wave owns a live cell q
#pragma unroll
            for (int q = 0; q < kCellsPerThread; ++q) wave_has[q] = __ballot(live[q]) != 0ull;
            float part[kCellsPerThread][kRedU];
#pragma unroll
            for (int q = 0; q < kCellsPerThread; ++q)
                if (wave_has[q]) {
#pragma unroll
                    for (int u = 0; u < kRedU; ++u) part[q][u] = lds.red[(t_of[q] << cp_log) + c + u * g_stride];
                }
#pragma unroll
            for (int q = 0; q < kCellsPerThread; ++q) {
                const bool fresh = d0 + t_of[q] * S >= 0 || at_start;   // first input row of the row is new
                sum[q] = fresh ? bias_c : ringv[q];
                if (wave_has[q]) {
#pragma unroll
                    for (int u = 0; u < kRedU; ++u) sum[q] += part[q][u];    // fixed order
                }
            }
            for (int gi = kRedU; gi < n_red; gi += kRedU) {   // the number of groups is a multiple of kRedU
#pragma unroll
                for (int q = 0; q < kCellsPerThread; ++q)
                    if (wave_has[q]) {
#pragma unroll
                        for (int u = 0; u < kRedU; ++u) part[q][u] = lds.red[(t_of[q] << cp_log) + c + (gi + u) * g_stride];
                    }
#pragma unroll
                for (int q = 0; q < kCellsPerThread; ++q)
                    if (wave_has[q]) {
#pragma unroll
                        for (int u = 0; u < kRedU; ++u) sum[q] += part[q][u];
                    }
            }
        }
        unsigned long long nzb[kCellsPerThread];
#pragma unroll
        for (int q = 0; q < kCellsPerThread; ++q) {
            bool emitted_nz = false;
            if (live[q]) {
                if (t_of[q] < t_fin) {
                    const float h = act == IDF_ACT_NONE ? sum[q] : fmaxf(sum[q], 0.f);
                    if (last) {
                        int64_t slot = ka.out_slot0[seg] + (t_of[q] - t_lo);
                        if (slot >= ka.out_cap) slot -= ka.out_cap;
                        ((gfloat *)ka.out)[(int64_t)stream * ka.out_stride + slot * c_out + c] = h;
                    } else if (hand_over) {
                        tr[(t_of[q] - t_lo) * c_out + c] = h;  // the next stage takes it up in the next launch
                    } else if (h != 0.f) {
                        xn[c * kXStride + (t_of[q] - t_lo)] = h;
                        emitted_nz = true;
                    }
                } else {
                    ringg[at[q]] = sum[q];                    // stays in the rolling buffer: in memory,
                    lds.ring[l][at[q]] = sum[q];              // and here for the launch's next segment
                }
            }
            nzb[q] = more ? __ballot(emitted_nz) : 0ull;
        }
        // The non-zero values just emitted are the next layer's events: their channels get their
        // bits now; the ballots are kept and counted after the chain.
        if (more && lane == 0) {
#pragma unroll
            for (int q = 0; q < kCellsPerThread; ++q) lds.nzlog[l][tid >> 6][q] = nzb[q];
            unsigned long long any_nz = 0;
#pragma unroll
            for (int q = 0; q < kCellsPerThread; ++q) any_nz |= nzb[q];
            if (any_nz) {
                const unsigned long long chans = fold_channels(any_nz, m.cp);
                if ((uint32_t)chans) atomicOr(&lds.chmask[cur_buf ^ 1][0], (uint32_t)chans);
                if ((uint32_t)(chans >> 32)) atomicOr(&lds.chmask[cur_buf ^ 1][1], (uint32_t)(chans >> 32));
            }
        }
        lds_barrier();
        cur_buf ^= 1;
    }

    // Events and executed taps of layers 1..: one lane per kept ballot (layer, wave, cell).  A
    // wave's ballot covers 64 / cp consecutive new rows of the layer before, cp lanes each.
    if (ka.stats && tid < (le - 1 - lb) * (kT / 64) * kCellsPerThread) {
        const int l = lb + tid / ((kT / 64) * kCellsPerThread), r = tid - (l - lb) * ((kT / 64) * kCellsPerThread);
        const int wv = r / kCellsPerThread, q = r - wv * kCellsPerThread;
        if (a.step[seg][l].cnt > 0 && a.step[seg][l + 1].cnt > 0) {
            const unsigned long long nz = lds.nzlog[l][wv][q];
            if (nz) {
                const int cp_log = a.layer[l].cp_log, cp = 1 << cp_log;
                const int j0 = ((wv * 64) >> cp_log) + q * (kT >> cp_log);
                const unsigned long long rowmask = cp == 64 ? ~0ull : ((1ull << cp) - 1ull);
                unsigned int ev = 0, taps = 0;
                for (int rr = 0; rr < (64 >> cp_log); ++rr) {
                    const int n = __popcll((nz >> (rr << cp_log)) & rowmask);
                    if (n) { ev += n; taps += n * cascade_taps(a.step[seg][l + 1], j0 + rr); }
                }
                unsigned long long *dst = ka.stats + ((int64_t)stream * n_layers + l + 1) * 2;
                atomicAdd(dst, (unsigned long long)ev);
                atomicAdd(dst + 1, (unsigned long long)taps * a.layer[l + 1].c_out);
            }
        }
    }
    if (seg + 1 < n_seg) {
        // The next segment starts in x[0] with clear channel bits.  Whatever this segment left in
        // the two row buffers is no longer read (every layer ended in a barrier), and the weights in
        // flight are the first channels of the stage's first layer again: the last layer a segment
        // reaches asks for them in its tail, a segment that reached none has left them untouched.
        for (int i = tid; i < 64 * kXStride / 4; i += kT) reinterpret_cast<float4 *>(lds.x[0])[i] = float4{0.f, 0.f, 0.f, 0.f};
        if (tid < 4) lds.chmask[tid >> 1][tid & 1] = 0;
        lds_barrier();
    }
    }   // segments
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
    static hipError_t prepared = [] {
        const void *kernels[4] = {reinterpret_cast<const void *>(k_cascade1d<false, 1>), reinterpret_cast<const void *>(k_cascade1d<true, 1>),
                                  reinterpret_cast<const void *>(k_cascade1d<false, kCasStepMax>), reinterpret_cast<const void *>(k_cascade1d<true, kCasStepMax>)};
        for (const void *k : kernels) {
            hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Lds));
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }();
    if (prepared != hipSuccess) return prepared;
    CascadeArgs b = a;
    // The stages are dealt to the eight XCDs when their number divides eight; a number that does
    // not is filled up with empty stages (their workgroups return at once).
    int grid_stages = b.n_stages;
    for (int d = 1; d <= 8 && d <= kCasMaxStages; d *= 2)
        if (d >= b.n_stages) { grid_stages = d; break; }
    const bool spread = 8 % grid_stages == 0 && sel.n % (8 / grid_stages) == 0;
    if (!spread) grid_stages = b.n_stages;
    for (int k = 0; k < grid_stages; ++k) {
        if (k < b.n_stages) { b.first[k] = b.layer[b.stage_lo[k]]; b.first_step[k] = b.step[0][b.stage_lo[k]]; }
        else { b.first[k] = CascadeLayer{}; b.first_step[k] = CascadeStep{}; b.stage_steps[k] = 0; }      // nothing to do
    }
    b.per = spread ? 8 / grid_stages : sel.n;
    if (sel.n / b.per > 65535) return hipErrorInvalidValue;
    // the variant that adds up what it issues is a kernel of its own: the one that is timed carries none of it
    const dim3 grid(b.per, grid_stages, sel.n / b.per), block(kCasThreads);
    if (b.steps_max <= 1) {
        // one step per stage (a launch per push): the short argument block, a third of the bytes to hand over and to sweep on chip
        CascadeArgsT<1> s1;
        memcpy(&s1, &b, sizeof(s1));
        if (b.issued) return launch(k_cascade1d<true, 1>, grid, block, sizeof(Lds), lc, s1, sel);
        return launch(k_cascade1d<false, 1>, grid, block, sizeof(Lds), lc, s1, sel);
    }
    if (b.issued) return launch(k_cascade1d<true, kCasStepMax>, grid, block, sizeof(Lds), lc, b, sel);
    return launch(k_cascade1d<false, kCasStepMax>, grid, block, sizeof(Lds), lc, b, sel);
}

}  // namespace idf
