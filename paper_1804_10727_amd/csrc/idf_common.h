// Shared between the host side of the library and its kernels: layer geometry, the
// data-independent row schedule, and the argument blocks handed to the kernels.
#pragma once

#include <stddef.h>
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define IDF_HD __host__ __device__ inline
#else
#define IDF_HD inline
#endif

namespace idf {

constexpr int kMaxLayers = 32;
constexpr int kSelIds = 16;    // stream ids carried by value in one launch (kept small: kernel arguments are fetched from memory)

struct Geom {
    int kind;            // IDF_CONV / IDF_MAXPOOL
    int c_in, c_out, k_h, k_w, s_h, s_w, p_h, p_w;
    int act, shr, clamp_hi;
    int h_in, w_in;      // h_in = 0: unbounded
    int h_out, w_out;    // h_out = 0: unbounded
};

IDF_HD int out_size(int n, int k, int s, int p)
{
    int t = n + 2 * p - k;
    return t < 0 ? 0 : t / s + 1;
}

// Number of output rows of a layer that are final once it has received rows 0..y-1 of its
// input.  Output row o needs input rows o*s-p .. o*s-p+k-1 (clipped to the sample), so it is
// final when y >= o*s-p+k, and every row is final once the whole sample (h_in rows) is in:
// the bottom padding contributes nothing.
IDF_HD int64_t rows_final(const Geom &g, int64_t y)
{
    if (g.h_in > 0 && y >= g.h_in) return g.h_out;
    int64_t t = y + g.p_h - g.k_h;
    int64_t n = t < 0 ? 0 : t / g.s_h + 1;
    if (g.h_out > 0 && n > g.h_out) n = g.h_out;
    return n;
}

// One past the last output row that input rows 0..y-1 have contributed to (first input row
// of output row o is o*s-p).
IDF_HD int64_t rows_touched(const Geom &g, int64_t y)
{
    if (y <= 0) return 0;
    int64_t n = (y - 1 + g.p_h) / g.s_h + 1;
    if (g.h_out > 0 && n > g.h_out) n = g.h_out;
    return n;
}

// Stream selection of one launch: either the contiguous ids base .. base+n-1 or n ids by value.
struct StreamSel {
    int n;
    int base;            // >= 0: contiguous; -1: use ids[]
    int pos0;            // position of the first selected stream in the caller's id list
    int ids[kSelIds];
};

__host__ __device__ inline int sel_stream(const StreamSel &s, int i) { return s.base >= 0 ? s.base + i : s.ids[i]; }

// One step of one conv layer for a group of streams that are all at the same row:
// input rows [y0, y0+cnt) arrive; output rows [o_lo, o_hi) are touched; of those
// [o_lo, o_fin) become final and are emitted, the rest go back to the ring.
struct ConvStep {
    Geom g;
    int layer;
    int64_t y0;
    int cnt;
    int64_t o_lo, o_fin, o_hi;
    int ring_rows;               // slots of the ring (k_h)
    // input rows: [stream or position][row - in_row0][w_in][c_in]
    const void *in;
    int64_t in_stream_stride;    // elements
    int64_t in_row0;             // input row held in slot 0
    int in_by_position;          // 1: index by position in the caller's list (network input)
    // state ring [stream][slot][w_out][c_out], slot = o mod ring_rows
    void *ring;
    int64_t ring_stream_stride;
    // destination of emitted rows: next layer's transit rows (slot = o - dst_row0) or, for the
    // last layer, the output area (slot = (dst_slot0 + o - dst_row0) mod out_cap)
    void *dst;
    int64_t dst_stream_stride;
    int64_t dst_row0, dst_slot0;
    int to_output;
    int64_t out_cap;
    const void *w;               // [k_h][k_w][c_in][c_out]
    const void *bias;            // [c_out] or null
    unsigned long long *stats;   // [stream][layer][2]: events_in, macs
    int n_layers;
    int tile_x, tile_c, cells_per_thread;
    // A pixel segment of the network input (one row, cnt == 1): only columns [x_lo, x_hi) of the row are there,
    // column x_lo first in the buffer; x_hi == 0: the whole row.  cont: an earlier segment of the same row has
    // started the rows it touches, so every cell continues from the ring.
    int x_lo, x_hi, cont;
};

struct PoolStep {
    Geom g;
    int layer;
    int64_t y0;
    int cnt;
    int64_t o_lo, o_fin;         // output rows emitted: [o_lo, o_fin)
    int hold_new;                // 1: the last new row is the even row of a pair: hold it
    const void *in;
    int64_t in_stream_stride;
    int64_t in_row0;
    int in_by_position;
    void *held;                  // [stream][w_in][c]
    int64_t held_stream_stride;
    void *dst;
    int64_t dst_stream_stride;
    int64_t dst_row0, dst_slot0;
    int to_output;
    int64_t out_cap;
    unsigned long long *stats;
    int n_layers;
};

// Whole-net cascade for 1-D nets (one launch per push).
constexpr int kCasThreads = 256;     // four waves: two workgroups share a CU
constexpr int kCasKMax = 9;        // kernel height at most
constexpr int kCasRowsMax = 16;    // rows a layer receives per push at most
constexpr int kCasMaxLayers = 8;
constexpr int kCasSlotsMax = kCasRowsMax + kCasKMax - 1;   // output rows a layer touches per push at most
constexpr int kCasAhead = 4;       // input channels whose weights are in flight per lane

// Lanes of the cascade's workgroup take the output channels (padded to a power of two) and
// split the input channels round-robin over the kCasThreads / pad groups that result; every
// lane runs the same number of steps, a multiple of kCasAhead, and the weight packing is
// zero padded to the input channels those steps reach.
IDF_HD int cascade1d_steps(int c_in, int c_out)
{
    int cp = 1;
    while (cp < c_out) cp *= 2;
    const int n_grp = kCasThreads / cp;
    const int n_q = (c_in + n_grp - 1) / n_grp;
    return (n_q + kCasAhead - 1) / kCasAhead * kCasAhead;
}
IDF_HD int cascade1d_cin_pad(int c_in, int c_out)
{
    int cp = 1;
    while (cp < c_out) cp *= 2;
    return kCasThreads / cp * cascade1d_steps(c_in, c_out);
}

// What a cascade launch needs to know of a layer whatever the segment.
struct CascadeLayer {
    int cp_log;              // log2 of c_out rounded up to a power of two
    int c_in, c_out, k_h, s_h, act;
    int steps;               // cascade1d_steps(c_in, c_out)
    int ring_floats;         // k_h * c_out
    int rcp_k;               // ceil(65536 / k_h): (v * rcp_k) >> 16 == v / k_h for the small v that occur
    const void *w;           // cascade packing, see cascade1d_weight_index
    const void *bias;
    void *ring;              // this launch's first stream is at ring + stream * ring_stride floats
    int64_t ring_stride;
};

// One step of one layer, in small integers: the new input rows of one pushed segment or of
// several consecutive ones taken together.  Accumulator slot t stands for output row o_base + t.
struct CascadeStep {
    signed char cnt;             // new input rows (0: the layer does not fire)
    signed char t_lo, t_fin, t_hi;   // slots [t_lo, t_hi) are live; those below t_fin become final
    signed char d0;              // first input row of slot 0 minus the first new row
    signed char at_start;        // 1: the first new row is row 0 of the sample
    signed char rho;             // (first new row + padding) mod stride
    signed char slot0;           // ring slot of accumulator slot 0 (slot of t is (slot0 + t) mod k_h)
    signed char seg0, seg_rows;  // first layer of stage 0: the new rows are seg_rows rows each of the pushed segments seg0, seg0 + 1, ...
    short fma_per_channel;       // multiply-adds a lane issues for one input channel that holds an event (all rows, all taps)
    short in_off, out_off;       // rows: where a stage's first layer finds its rows in the hand-over buffer of the stage before,
                                 // and where its last layer puts the rows it hands over (both counted from the launch's first row)
    unsigned char taps4[kCasRowsMax / 2];   // per new row, four bits each: kernel taps landing inside the output
};
IDF_HD int cascade_taps(const CascadeStep &s, int j) { return (s.taps4[j >> 1] >> ((j & 1) * 4)) & 15; }

// The layers can be dealt to up to kCasMaxStages groups of workgroups (blockIdx.y) that run side
// by side in one launch, stage s working on the segments pushed s launches earlier: its first
// layer reads what stage s-1 wrote in the launch before (double-buffered by launch parity).
// A launch can take several segments of every stream at once (segments pushed in step and held
// back until there are enough of them): a stage then takes as many consecutive ones together as
// fit the rows one step can take, and runs the resulting steps one after the other with its
// layers' rolling buffers staying in LDS in between.
constexpr int kCasMaxStages = 8;
constexpr int kCasSegMax = 16;       // pushed segments one launch can take
constexpr int kCasStepMax = 8;       // steps a stage runs in one launch

// (NSTEP: steps of room in the block; a launch of one step per stage passes the short form, whose fields lie where the long one's do)
template <int NSTEP> struct CascadeArgsT {
    int n_layers;
    int n_stages;
    int stage_lo[kCasMaxStages + 1];     // stage s runs layers [stage_lo[s], stage_lo[s+1])
    int stage_steps[kCasMaxStages];      // steps stage s runs in this launch (0: nothing has reached it)
    int steps_max;                       // the largest of them
    int transit_wr;                      // parity of the hand-over buffers written by this launch
    int per;                             // filled by the launcher: streams side by side in blockIdx.x
    CascadeLayer layer[kCasMaxLayers];
    CascadeLayer first[kCasMaxStages];   // filled by the launcher: first[s] = layer[stage_lo[s]], first_step[s] = step[0][stage_lo[s]],
    CascadeStep first_step[kCasMaxStages];   // so that a workgroup finds them from its stage alone, in its first round of loads
    const void *in[kCasSegMax];          // stage 0: pushed segment q as [position][rows][c0]
    int in_stream_stride[kCasSegMax];    // elements
    void *transit;                       // hand-over rows [boundary][parity][stream][row][channel]
    int64_t transit_stream_stride, transit_buf_stride;   // floats
    void *out;                           // output area [stream][out_cap][c_out]
    int64_t out_stride, out_cap;
    int64_t out_slot0[kCasStepMax];      // of the steps the last stage runs
    unsigned long long *stats;
    unsigned long long *issued;          // [stream][layer]: multiply-adds issued (all rows of every channel that holds an event)
    CascadeStep step[NSTEP][kCasMaxLayers];   // step[m][l]: step m of layer l's stage (last in the block)
};
using CascadeArgs = CascadeArgsT<kCasStepMax>;

// One arriving row of a 3x3 / stride 1 / same-padded conv layer on the matrix cores.
// Tap ky of input row y lands on output row o = y + 1 - ky.
enum { kEmitNone = 0,      // row not final: back to the rolling buffer
       kEmitDirect,        // final: activate and emit
       kEmitHold,          // final, even row of a pool pair: becomes the pool's held row
       kEmitPoolHeld,      // final, odd row of a pool pair: max with the held row, emit pooled row
       kEmitPoolReg,       // final, odd row whose even partner became final in the same launch
       kEmitKeep };        // not final, and the step's second input row follows at once: stays in the accumulators
enum { kMfmaTile64x64 = 0, kMfmaTile128x32, kMfmaTile32x64, kMfmaTile32x32, kMfmaTile64x32 };

struct MfmaTap {
    int valid;             // output row exists
    int fresh;             // first touched by this input row: starts from the bias
    int emit;              // kEmit*
    int store_held;        // kEmitHold: write the held row (not needed when its partner follows at once)
    int ring_slot;
    int64_t dst_slot;      // row slot in the destination (pooled row slot for the pool cases)
};

struct MfmaStep {
    int w, c_in, c_out, c_out_pad;
    unsigned c_in_rcp;                 // ceil(2^32 / c_in): k / c_in = umulhi(k, c_in_rcp) for the k in use
    unsigned chunks_rcp;               // the same for the 16-byte cells per position (0: fewer channels than a cell)
    int act, shr, clamp_hi;
    int layer, pool_layer, n_layers;   // pool_layer < 0: no fused pool
    int taps_y;                        // taps of this input row that land inside the output (for the counters)
    int x_lo, x_hi;                    // columns of the input row that are given (a pixel segment); the rest reads as zero
    int skip_clear_tiles;              // tiles no given column reaches have nothing to do (no row starts or ends)
    int tile;                          // kMfmaTile*
    MfmaTap t[3];
    int dbl;                           // the step takes a second input row straight after the first (batch launches only):
    int taps_y2;                       //   its taps_y, its tap rows (rows y and y+1 arrive in the accumulators), its place
    MfmaTap t2[3];
    int64_t in_row_off2;
    const void *in;                    // input rows
    int64_t in_stream_stride, in_row_off;   // elements
    int in_by_position;
    void *ring;  int64_t ring_stream_stride;
    void *held;  int64_t held_stream_stride;
    void *dst;   int64_t dst_stream_stride;
    int to_output;
    const void *wfrag;                 // fragment-ordered weights
    const void *w_ev;                  // int8 nets: weights for the event path, [kx][c_in][c_out_pad] words of the three ky taps
    int ev_limit;                      // a tile with at most this many events (its halo included) goes the event path (0: never)
    const void *bias;
    unsigned long long *stats;
    unsigned long long *issued;        // [stream][layer]: multiply-adds issued by the matrix instructions (zeros inside live steps included)
};

// Steps of several layers for one launch of the matrix-core kernel.
constexpr int kMfmaBatchMax = 8;
struct MfmaBatch {
    int n;
    int tile;                          // kMfmaTile* (not 128x32), the same for every step
    MfmaStep st[kMfmaBatchMax];
};
static_assert(sizeof(MfmaBatch) + sizeof(StreamSel) <= 4096, "a launch's arguments must fit the kernel-argument segment");

struct CopyOut {
    const void *src;             // output area [stream][out_cap][row_elems]
    int64_t src_stream_stride;
    int64_t out_cap;
    void *dst;                   // [position][max_rows][row_elems]
    int64_t dst_stream_stride;
    int64_t row_elems;
    int elem_bytes;
};

// One layer's step in eager emission: output rows [o_lo, o_hi) take in the delta rows
// [i_lo, i_hi) of the layer before.  Per stream every level (0 = the input) keeps rows of 4-byte
// values [rows kept][W][C]: state c (conv layers), announced value, and the deltas it emitted for
// the segment in flight.  Row r lies in slot r mod (rows kept): a ring of the rows that can still
// change or be looked at (the cone of Sec. 3), or the whole map when as many rows are kept as the
// level has.
struct EagerStep {
    Geom g;                      // unused for the input step
    int layer, n_layers;
    int o_lo, o_hi, i_lo, i_hi;
    int w_out, c_out;            // input step: shape of an input row
    int init_bias;               // the state starts from the bias (first pass of a sample)
    int fresh_lo;                // rows >= fresh_lo of this level are reached for the first time: state and
                                 // announced value start from zero whatever their slots hold
    int in_hi;                   // rows >= in_hi of the level before have not been reached yet: they read as zero
    int round_bf16;              // announced values are rounded to bfloat16 (events of a bfloat16 net)
    int in_rows, c_rows, ann_rows, dlt_rows;   // rows kept: of the level before (announced and deltas alike), of this level's maps
    const void *in;              // input step: pushed rows [position][rows][w][c], event type
    int64_t in_stream_stride;
    const void *dlt_in, *ann_in; // maps of the layer before
    int64_t in_map_stride;       // elements per stream of those
    void *c, *ann, *dlt_out;     // this layer's maps
    int64_t c_stride, ann_stride, dlt_stride;   // elements per stream
    const void *w, *bias;
    unsigned long long *stats;
};

// Averaging output units: rows [first_slot, first_slot + n_rows) of the output ring are added to
// the per-channel sums of each selected stream.
struct HeadAcc {
    const void *src;             // output area [stream][out_cap][w][c], 4-byte elements
    int64_t src_stream_stride;
    int64_t out_cap;
    int w, c;
    int is_int;                  // elements are int32 (else float32)
    int zero_first;              // the sums start anew with these rows
    double count;                // positions averaged once these rows are in
    double *sums, *mean;         // [stream][c] each
};

// Fully connected output units over the last layer's map: rows [first_slot, first_slot + n_rows)
// of the output ring, which are rows row0 .. of the sample, are added, weighted, to every unit.
struct HeadUnits {
    const void *src;             // output area [stream][out_cap][w][c], 4-byte elements
    int64_t src_stream_stride;
    int64_t out_cap;
    int w, c, n_units;
    int is_int;
    int zero_first;              // the units start anew (from their bias) with these rows
    int64_t row0;
    int64_t map_elems;           // out_h * w * c: weights of one unit
    const float *weights;        // [unit][out_h][w][c]
    const float *bias;           // [unit] or null
    double *values;              // [stream][unit]
};

}  // namespace idf
