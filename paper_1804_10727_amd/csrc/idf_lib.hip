// Host side of the library: network description, workspace layout, the data-independent
// row schedule of a push (which layer receives which rows, which rows become final), and the
// kernel launches.  All arithmetic of the method runs in the kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <tuple>
#include <vector>

#include "idf.h"
#include "idf_common.h"
#include "idf_kernels.h"

using namespace idf;

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

// Workspace of idf_open_streams_static: one array per GPU, living in the library's code object
// until the process ends.  Its name is only a handle on the host side; the device address is
// asked for once per device (scratch_of) and only that pointer is ever handed to kernels, fills
// and copies.
constexpr size_t kStaticScratchBytes = (size_t)IDF_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
struct StaticScratch { unsigned char *ptr = nullptr; bool in_use = false; };
StaticScratch g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

int ev_bytes(int prec) { return prec == IDF_PREC_F32 ? 4 : prec == IDF_PREC_BF16 ? 2 : 1; }
int w_bytes(int prec) { return ev_bytes(prec); }

}  // namespace

struct idf_net {
    int precision = 0;
    int in_h = 0, in_w = 0, in_c = 0;
    std::vector<Geom> g;
    // device images: per conv layer weights [k_h][k_w][c_in][c_out] and bias [c_out] (4-byte)
    std::vector<std::vector<unsigned char>> w_img, b_img;
    // per conv layer the matrix-core kernel can serve: weights in its fragment order (else empty)
    std::vector<std::vector<unsigned char>> wm_img;
    int out_w = 0, out_c = 0;
    int64_t out_h = 0;
    int open_count = 0;
};

struct StreamHost {
    int64_t r = 0;            // rows of the current sample received
    int64_t out_written = 0;  // output rows completed since open/reset
    int64_t out_read = 0;     // output rows handed over
    int64_t head_done = 0;    // output rows the averaging units have taken in
    int64_t head_base = 0;    // first of the rows they average (start of the current sample)
    int x_next = 0;           // columns of the current row received (pixel segments)
    int64_t eager_rows = 0;   // eager emission: input rows of the sample last presented that the levels have seen
};

struct ProfRec {
    int kind, layer;
    hipEvent_t a, b;
    double bytes;
};

struct idf_streams {
    int static_dev = -1;             // >= 0: the workspace is that device's static array (given back at close)
    int cus = 0;                     // compute units of the device the streams were opened on
    int ev_per_step = 0;             // int8 event path (idf_set_event_path): events a tile may hold per K-step of its contraction and still go that way; 0: off
    bool use_cascade1d = false;      // whole-net kernel for 1-D nets instead of one launch per layer
    bool prof_on = false;
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> ev_pool;
    idf_net *net = nullptr;
    int B = 0, max_seg = 0;
    int64_t out_cap = 0;
    hipStream_t st = nullptr;
    char *ws = nullptr;
    size_t ws_bytes = 0;
    std::vector<size_t> w_off, b_off, wm_off, ring_off, held_off, transit_off;
    std::vector<int> mfma;           // per layer: 1 = matrix-core conv kernel, 2 = pool fused into the conv before it
    std::vector<int64_t> ring_stride, held_stride, transit_stride;   // elements per stream
    std::vector<int> transit_cap;                                    // rows per stream
    size_t out_off = 0, stats_off = 0, issued_off = 0, head_off = 0;
    bool count_issued = false;       // the kernels add up what they issue (an atomic per wave: switched on for measurements)
    bool head_on = false;
    int head_units = 0;              // fully connected output units (0: only the averaging units)
    char *head_units_ws = nullptr;   // caller's buffer: weights [unit][map], bias [unit], values [stream][unit]
    bool head_units_bias = false;
    int64_t out_stride = 0;
    std::vector<std::vector<float>> cas_w;      // cascade packing of the weights (kept until the upload has run)
    // 1-D cascade, layers dealt to stages that run side by side, stage k on the segments of the
    // launch k launches earlier: the launches still on their way, newest first.  A launch holds
    // one segment of every stream, or up to cas_batch of them when pushes in step are held back
    // (idf_set_push_batching); cas_pending are the segments waiting for their launch.
    struct CasSeg {
        int64_t y0[kCasMaxLayers + 1];       // per layer: first of the rows the segment brings it (entry n_layers: first output row)
        int cnt[kCasMaxLayers + 1];          // and how many
        int64_t out_slot0 = 0; const void *dev_rows = nullptr; int n_rows = 0;
    };
    struct CasGroup {                                                            // n = 0: none
        int n = 0; double bytes = 0; CasSeg seg[kCasSegMax];
        void take(const CasGroup &o) { n = o.n; bytes = o.bytes; for (int q = 0; q < o.n; ++q) seg[q] = o.seg[q]; }
    };
    int cas_stages = 1;
    int cas_lo[kCasMaxStages + 1] = {};
    CasGroup cas_ring[kCasMaxStages];        // the launches on their way: the one k launches back is hist(k - 1)
    int cas_head = 0;
    CasGroup &hist(int k) { return cas_ring[(cas_head + k) % kCasMaxStages]; }
    CasGroup cas_pending;
    int cas_batch = 1;
    CascadeLayer cas_layer[kCasMaxLayers];
    int cas_parity = 0;
    size_t cas_transit_off = 0;
    int64_t cas_transit_stride = 0;
    // 2-D nets served by the matrix-core kernel throughout: one launch per arriving row holds a
    // step of every conv layer, each on a row that was complete before the launch.  Per conv
    // layer ("unit") the rows waiting for it, and where in the ring of hand-over rows they lie.
    struct StgRow { int64_t y; int slot; };
    bool stg2d = false;
    std::vector<std::pair<int, int>> push_members;   // (position, id) of the streams of the push being checked
    std::vector<int> stg_unit;                  // conv layer of unit k
    std::vector<std::deque<StgRow>> stg_fifo;
    std::vector<int64_t> stg_seq;               // rows emitted by unit k so far
    int64_t stg_out_next = 0;                   // output slot of the next completed row
    int stg_tile = kMfmaTile64x64;              // tile shape of the staged launches
    int stg_slots = 4;                          // rows of a hand-over ring (kStgSlots, twice that where a step may take two rows)
    bool stg_pairs = false;                     // pushes of several rows go through the layers two rows per launch
    // eager emission: per stream and level (0 = input) rows of state, announced values and deltas in a
    // workspace of its own -- rings of the rows that can still change or be looked at (nets without
    // biases) or whole maps
    struct Eager {
        bool on = false;
        bool ring = false;
        char *ws = nullptr;
        std::vector<int64_t> row_elems;           // per level: W*C of one row
        std::vector<int> rows;                    // per level: rows the level has (H)
        std::vector<int> ann_rows, cd_rows;       // per level: rows kept of the announced values / of state and deltas
        std::vector<size_t> ann_off, c_off, dlt_off;   // per level (c: conv layers only)
    } eager;
    // a pixel segment being pushed: columns [x_lo, x_hi) of the current row of layer 0 (else the whole row)
    struct Part { bool on = false; int x_lo = 0, x_hi = 0; bool first = true, last = true; } part;
    std::vector<StreamHost> h;
    std::vector<int> stamp;
    int stamp_gen = 0;
    idf_sizes sizes{};
};

namespace {

// Rows the last layer completes when a stream at row r receives n more rows.
int64_t output_rows_of_push(const idf_net &net, int64_t r, int n)
{
    int64_t y0 = r, cnt = n;
    for (const Geom &g : net.g) {
        int64_t a = rows_final(g, y0), b = rows_final(g, y0 + cnt);
        y0 = a;
        cnt = b - a;
        if (cnt == 0) return 0;
    }
    return cnt;
}

// Most rows a layer can emit in one step when it receives at most cap_in rows.
int max_emit(const Geom &g, int cap_in)
{
    int64_t best = 0;
    auto probe = [&](int64_t y0) {
        if (y0 < 0) return;
        int64_t cnt = cap_in;
        if (g.h_in > 0) {
            if (y0 >= g.h_in) return;
            cnt = std::min<int64_t>(cnt, g.h_in - y0);
        }
        best = std::max(best, rows_final(g, y0 + cnt) - rows_final(g, y0));
    };
    int64_t span = (int64_t)4 * g.k_h * g.s_h + cap_in + 4;
    for (int64_t y0 = 0; y0 <= span; ++y0) probe(y0);
    if (g.h_in > 0)
        for (int64_t y0 = g.h_in - span; y0 < g.h_in; ++y0) probe(y0);
    return (int)best;
}

struct Layout {
    std::vector<size_t> w_off, b_off, wm_off, ring_off, held_off, transit_off;
    std::vector<int64_t> ring_stride, held_stride, transit_stride;
    std::vector<int> transit_cap;
    size_t out_off = 0, stats_off = 0, issued_off = 0, head_off = 0, total = 0;
    int64_t out_stride = 0;
    bool cascade1d = false;          // the whole-net 1-D kernel serves this stream set
    size_t cas_transit_off = 0;      // hand-over rows between the cascade's stages
    int64_t cas_transit_stride = 0;  // floats per stream in one hand-over buffer
    int cas_boundaries = 0;          // stage boundaries the block has room for
    idf_sizes sizes{};
};

// Staged layers (one launch per arriving row, layer l a launch behind layer l-1): rows a layer has
// completed wait for the next layer's step in a small ring per layer and stream.  The host never
// leaves more than kStgWait rows waiting per layer when a call returns; a launch reads one slot,
// leaves at most kStgWait - 1 waiting and writes at most two new rows, hence kStgSlots.
constexpr int kStgWait = 2;
constexpr int kStgSlots = 4;

// The layers run strictly depth-first within each call (nothing waits between layers across
// calls) when the staged modes are switched off.
bool strict_rows() { return getenv("IDF_NO_MFMA") || getenv("IDF_NO_ROW_STAGES"); }
bool strict_cascade() { const char *e = getenv("IDF_CASCADE_STAGES"); return e && atoi(e) <= 1; }

// Every conv layer can run on the matrix-core kernel and every pool is fused behind one.
bool net_all_mfma(const idf_net &net)
{
    const int n = (int)net.g.size();
    int units = 0;
    for (int l = 0; l < n; ++l) {
        if (net.g[l].kind == IDF_CONV) {
            if (net.wm_img[l].empty()) return false;
            ++units;
        } else if (l == 0 || net.g[l - 1].kind != IDF_CONV || net.g[l].k_w != 2) {
            return false;
        }
    }
    return units >= 1 && units <= kMfmaBatchMax;
}

int make_layout(const idf_net &net, int B, int max_seg, int64_t out_cap, Layout &L)
{
    const int n = (int)net.g.size();
    const int eb = ev_bytes(net.precision);
    size_t off = 0;
    L.w_off.assign(n, 0); L.b_off.assign(n, 0); L.wm_off.assign(n, 0);
    L.ring_off.assign(n, 0); L.held_off.assign(n, 0); L.transit_off.assign(n, 0);
    L.ring_stride.assign(n, 0); L.held_stride.assign(n, 0); L.transit_stride.assign(n, 0);
    L.transit_cap.assign(n, 0);
    {
        int cap = max_seg;
        for (int l = 0; l < n; ++l) {
            cap = std::max(1, max_emit(net.g[l], cap));
            L.transit_cap[l] = cap;
        }
    }
    L.cascade1d = cascade1d_eligible(net.precision, net.g.data(), n, L.transit_cap.data(), max_seg);
    const bool all_mfma = net_all_mfma(net);
    for (int l = 0; l < n; ++l) {
        if (net.g[l].kind != IDF_CONV) continue;
        // the 1-D cascade reads its own packing, taps zero-padded to kCasKMax
        size_t wsz = net.w_img[l].size();
        if (L.cascade1d) wsz = (size_t)cascade1d_cin_pad(net.g[l].c_in, net.g[l].c_out) * net.g[l].c_out * kCasKMax * 4;
        L.w_off[l] = off; off = align_up(off + wsz);
        L.b_off[l] = off; off = align_up(off + net.b_img[l].size());
        L.wm_off[l] = off; off = align_up(off + net.wm_img[l].size());
    }
    L.sizes.weights_bytes = off;
    size_t state_per_stream = 0, transit_per_stream = 0, handover_per_stream = 0;
    const bool staged_rows = all_mfma && !strict_rows();
    int cap = max_seg;
    for (int l = 0; l < n; ++l) {
        const Geom &g = net.g[l];
        if (g.kind == IDF_CONV) {
            L.ring_stride[l] = (int64_t)g.k_h * g.w_out * g.c_out;
            L.ring_off[l] = off; off = align_up(off + (size_t)L.ring_stride[l] * 4 * B);
            state_per_stream += (size_t)L.ring_stride[l] * 4;
        } else {
            L.held_stride[l] = (int64_t)g.w_in * g.c_out;
            L.held_off[l] = off; off = align_up(off + (size_t)L.held_stride[l] * eb * B);
            state_per_stream += (size_t)L.held_stride[l] * eb;
        }
        cap = L.transit_cap[l];
        // (the 1-D cascade passes rows on inside LDS; a conv layer's rows go straight into a fused pool)
        const bool into_fused_pool = all_mfma && !getenv("IDF_NO_MFMA") && l + 1 < n && net.g[l + 1].kind == IDF_MAXPOOL;
        if (l < n - 1 && !L.cascade1d && !into_fused_pool) {
            // room for the hand-over ring when the layers are staged across pushes
            // (a step that takes two rows can complete three and reads two more meanwhile: twice the slots)
            const int rows = all_mfma ? std::max(cap, max_seg >= 2 ? 2 * kStgSlots : kStgSlots) : cap;
            L.transit_stride[l] = (int64_t)rows * g.w_out * g.c_out;
            L.transit_off[l] = off; off = align_up(off + (size_t)L.transit_stride[l] * eb * B);
            transit_per_stream += (size_t)L.transit_stride[l] * eb;
            // rows that can wait for the next conv layer when a call returns
            if (staged_rows) handover_per_stream += (size_t)kStgWait * g.w_out * g.c_out * eb;
        }
    }
    if (out_cap <= 0) {
        if (net.out_h <= 0) return fail(IDF_EINVAL, "an unbounded net needs out_cap_rows > 0");
        out_cap = net.out_h;
    }
    if (out_cap < L.transit_cap[n - 1])
        return fail(IDF_EINVAL, "out_cap_rows %lld is smaller than the %d rows one push can complete",
                    (long long)out_cap, L.transit_cap[n - 1]);
    L.out_stride = out_cap * net.out_w * net.out_c;
    L.out_off = off; off = align_up(off + (size_t)L.out_stride * 4 * B);
    L.stats_off = off; off = align_up(off + (size_t)B * n * 2 * sizeof(unsigned long long));
    L.issued_off = off; off = align_up(off + (size_t)B * n * sizeof(unsigned long long));
    L.head_off = off; off = align_up(off + (size_t)B * net.out_c * 2 * sizeof(double));   // sums, means
    if (L.cascade1d) {
        // Rows passed from one stage to the next, double-buffered by launch parity: room for a
        // boundary behind every layer but the last, each as large as the largest hand-over.
        int64_t most = 0;
        for (int l = 0; l < n - 1; ++l) {
            most = std::max<int64_t>(most, (int64_t)L.transit_cap[l] * net.g[l].c_out);
            // what is alive between two pushes if every layer is a stage of its own
            if (!strict_cascade()) handover_per_stream += (size_t)L.transit_cap[l] * net.g[l].c_out * 4;
        }
        L.cas_boundaries = std::min(kCasMaxStages, n) - 1;
        L.cas_transit_stride = (most + 63) / 64 * 64;          // of one segment; a launch can hold kCasSegMax of them
        L.cas_transit_off = off;
        off = align_up(off + (size_t)L.cas_boundaries * 2 * B * kCasSegMax * L.cas_transit_stride * 4);
        transit_per_stream = (size_t)L.cas_boundaries * 2 * kCasSegMax * L.cas_transit_stride * 4;
        // (a launch of held-back segments hands over the rows of all of them: kCasSegMax times the
        // rows of one; with a launch per push only the first of these is ever in use)
    }
    L.total = off;
    L.sizes.workspace_bytes = off;
    L.sizes.state_bytes_per_stream = state_per_stream;
    L.sizes.handover_bytes_per_stream = handover_per_stream;
    L.sizes.retained_bytes_per_stream = state_per_stream + handover_per_stream;
    L.sizes.transit_bytes_per_stream = transit_per_stream;
    L.sizes.output_bytes_per_stream = (size_t)L.out_stride * 4;
    L.sizes.out_w = net.out_w; L.sizes.out_c = net.out_c; L.sizes.out_h = net.out_h;
    return IDF_OK;
}

int check_ids(idf_streams *s, const int32_t *ids, int n_ids)
{
    if (n_ids < 1 || n_ids > s->B) return fail(IDF_EINVAL, "n_ids %d outside [1, %d]", n_ids, s->B);
    if (!ids) return IDF_OK;
    if (++s->stamp_gen == 0x7fffffff) { std::fill(s->stamp.begin(), s->stamp.end(), 0); s->stamp_gen = 1; }
    for (int i = 0; i < n_ids; ++i) {
        if (ids[i] < 0 || ids[i] >= s->B) return fail(IDF_EINVAL, "stream id %d outside [0, %d)", ids[i], s->B);
        if (s->stamp[ids[i]] == s->stamp_gen) return fail(IDF_EINVAL, "stream id %d given twice", ids[i]);
        s->stamp[ids[i]] = s->stamp_gen;
    }
    return IDF_OK;
}

// Splits a list of (position, id) pairs into launch selections: maximal runs that are
// contiguous in both position and id go by base, the rest by value in blocks of kSelIds.
template <class F> int for_each_selection(const std::vector<std::pair<int, int>> &members, F &&f)
{
    size_t i = 0;
    while (i < members.size()) {
        size_t j = i + 1;
        while (j < members.size() && members[j].first == members[j - 1].first + 1 &&
               members[j].second == members[j - 1].second + 1 && j - i < 65535)
            ++j;
        StreamSel sel{};
        if (j - i >= 2 || members.size() - i == 1) {
            sel.n = (int)(j - i); sel.base = members[i].second; sel.pos0 = members[i].first;
            int rc = f(sel);
            if (rc != IDF_OK) return rc;
            i = j;
            continue;
        }
        // by value: positions must still be consecutive within one selection
        j = i + 1;
        while (j < members.size() && members[j].first == members[j - 1].first + 1 && j - i < (size_t)kSelIds) ++j;
        sel.n = (int)(j - i); sel.base = -1; sel.pos0 = members[i].first;
        for (size_t k = i; k < j; ++k) sel.ids[k - i] = members[k].second;
        int rc = f(sel);
        if (rc != IDF_OK) return rc;
        i = j;
    }
    return IDF_OK;
}

int dev_fail(hipError_t e, const char *what)
{
    return fail(IDF_EDEVICE, "%s: %s", what, hipGetErrorString(e));
}

// Launch context of the next kernel: plain, or with a fresh event pair while profiling.
LaunchCtx launch_ctx(idf_streams *s, int kind, double bytes, int layer = -1)
{
    LaunchCtx c;
    c.st = s->st;
    if (!s->prof_on) return c;
    hipEvent_t ev[2] = {nullptr, nullptr};
    for (int i = 0; i < 2; ++i) {
        if (!s->ev_pool.empty()) { ev[i] = s->ev_pool.back(); s->ev_pool.pop_back(); }
        else if (hipEventCreate(&ev[i]) != hipSuccess) { ev[i] = nullptr; }
    }
    if (!ev[0] || !ev[1]) {            // out of events: run this launch unprofiled
        for (int i = 0; i < 2; ++i) if (ev[i]) s->ev_pool.push_back(ev[i]);
        return c;
    }
    c.start = ev[0]; c.stop = ev[1];
    s->prof.push_back(ProfRec{kind, layer, ev[0], ev[1], bytes});
    return c;
}

// Bytes one conv step has to move by the definition of the method: the new input rows, the
// retained rows of c it continues (read) and leaves unfinished (written), the rows it emits,
// per stream; the layer's weights once.
double conv_step_bytes(const idf_net &net, const ConvStep &a, int n_streams)
{
    const int eb = ev_bytes(net.precision);
    const double row_in = (double)a.g.w_in * a.g.c_in * eb, row_out = (double)a.g.w_out * a.g.c_out;
    const int64_t old_rows = std::max<int64_t>(0, std::min(rows_touched(a.g, a.y0), a.o_hi) - a.o_lo);
    // rows handed from layer to layer are not counted: the method does not require them to
    // leave the chip
    double per_stream = (a.in_by_position ? a.cnt * row_in : 0.0) + old_rows * row_out * 4 +
                        (double)(a.o_hi - a.o_fin) * row_out * 4 +
                        (a.to_output ? (double)(a.o_fin - a.o_lo) * row_out * 4 : 0.0);
    double weights = (double)a.g.k_h * a.g.k_w * a.g.c_in * a.g.c_out * w_bytes(net.precision) + (a.bias ? a.g.c_out * 4.0 : 0.0);
    return per_stream * n_streams + weights;
}

// Deals the cascade's layers to stages.  A stage costs a fixed part and a part per layer that
// grows with the layer's steps; the split with the cheapest slowest stage wins, as long as all
// workgroups of a launch (streams x stages) are resident at once, two to a compute unit.
void plan_cascade_stages(idf_streams *s)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    int cus = 0, dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        cus = 0;
    int max_stages = std::min({kCasMaxStages, n, std::max(1, 2 * cus / std::max(1, s->B))});      // two workgroups fit a CU
    if (const char *e = getenv("IDF_CASCADE_STAGES")) max_stages = std::max(1, std::min(max_stages, atoi(e)));
    if (strict_cascade()) max_stages = 1;
    std::vector<double> cost(n);
    for (int l = 0; l < n; ++l) cost[l] = 2.5 + 0.2 * cascade1d_steps(net.g[l].c_in, net.g[l].c_out);
    const double fixed = 4.0;
    // Contiguous groups of layers, at most max_stages of them, the slowest as fast as possible
    // (on a tie, fewer stages): best[k][i] = cost of the slowest of k stages over layers [0, i).
    std::vector<std::vector<double>> best(max_stages + 1, std::vector<double>(n + 1, 1e30));
    std::vector<std::vector<int>> cut(max_stages + 1, std::vector<int>(n + 1, 0));
    best[0][0] = 0;
    for (int k = 1; k <= max_stages; ++k)
        for (int i = k; i <= n; ++i) {
            double t = fixed;
            for (int j = i - 1; j >= k - 1; --j) {         // the last stage is layers [j, i)
                t += cost[j];
                const double w = std::max(best[k - 1][j], t);
                if (w < best[k][i]) { best[k][i] = w; cut[k][i] = j; }
            }
        }
    int best_n = 1;
    for (int k = 2; k <= max_stages; ++k)
        if (best[k][n] + 0.3 * k < best[best_n][n] + 0.3 * best_n) best_n = k;
    int best_lo[kCasMaxStages + 1];
    for (int k = 0; k <= kCasMaxStages; ++k) best_lo[k] = n;
    for (int k = best_n, i = n; k >= 1; --k) { i = cut[k][i]; best_lo[k - 1] = i; }
    s->cas_stages = best_n;
    for (int k = 0; k <= kCasMaxStages; ++k) s->cas_lo[k] = best_lo[k];
}

// What a cascade launch needs to know of every layer whatever the segment.
void cascade_layers(idf_streams *s)
{
    const idf_net &net = *s->net;
    for (int l = 0; l < (int)net.g.size() && l < kCasMaxLayers; ++l) {
        const Geom &g = net.g[l];
        CascadeLayer &L = s->cas_layer[l];
        L = CascadeLayer{};
        L.c_in = g.c_in; L.c_out = g.c_out; L.k_h = g.k_h; L.s_h = g.s_h; L.act = g.act;
        L.steps = cascade1d_steps(g.c_in, g.c_out);
        L.ring_floats = g.k_h * g.c_out;
        L.rcp_k = (65536 + g.k_h - 1) / g.k_h;
        L.w = s->ws + s->w_off[l];
        L.bias = net.b_img[l].empty() ? nullptr : s->ws + s->b_off[l];
        L.ring = s->ws + s->ring_off[l];
        L.ring_stride = s->ring_stride[l];
        L.cp_log = 0;
        while ((1 << L.cp_log) < g.c_out) ++L.cp_log;
    }
}

// Which rows a segment of n_rows rows arriving at row r brings to every layer.
void cascade_propagate(idf_streams *s, int n_rows, int64_t r, int n_streams, idf_streams::CasSeg &p, double &bytes)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    int64_t y0 = r, cnt = n_rows;
    for (int l = 0; l < n; ++l) {
        const Geom &g = net.g[l];
        p.y0[l] = y0; p.cnt[l] = (int)cnt;
        if (cnt > 0) {
            ConvStep c{};
            c.g = g; c.y0 = y0; c.cnt = (int)cnt; c.o_lo = rows_final(g, y0); c.o_fin = rows_final(g, y0 + cnt);
            c.o_hi = std::max(rows_touched(g, y0 + cnt), c.o_fin);
            c.in_by_position = l == 0; c.to_output = l == n - 1; c.bias = s->cas_layer[l].bias;
            bytes += conv_step_bytes(net, c, n_streams);
            y0 = c.o_lo; cnt = c.o_fin - c.o_lo;
        }
    }
    p.y0[n] = y0; p.cnt[n] = (int)cnt;
}

// The step of layer l for input rows [y0, y0 + cnt).
int cascade_step(const idf_net &net, int l, int64_t y0, int64_t cnt, CascadeStep &L)
{
    const Geom &g = net.g[l];
    L = CascadeStep{};
    if (cnt <= 0) return IDF_OK;
    const int64_t o_lo = rows_final(g, y0), o_fin = rows_final(g, y0 + cnt);
    const int64_t o_hi = std::max(rows_touched(g, y0 + cnt), o_fin);
    const int64_t y0p = y0 + g.p_h;
    const int rho = (int)(y0p % g.s_h);
    const int64_t o_base = y0p / g.s_h + cascade1d_slot_off(g.s_h, rho);
    {   // what a lane issues per channel that holds an event: the kernel's variant for 4, 8 or 16
        // new rows computes all of them, all nine tap positions that land on an output row
        // (the cascade takes strides 1 and 2 only: parity by mask, no division in what runs with every push)
        const int nin = cnt <= 4 ? 4 : cnt <= 8 ? 8 : 16, par = g.s_h - 1;
        int f = 0;
        for (int j = 0; j < nin; ++j)
            for (int ky = 0; ky < kCasKMax; ++ky)
                if (((rho + j - ky) & par) == 0) ++f;
        L.fma_per_channel = (short)f;
    }
    const int64_t t_lo = o_lo - o_base, t_fin = o_fin - o_base, t_hi = o_hi - o_base;
    const int64_t d0 = o_base * g.s_h - g.p_h - y0;
    if (cnt > kCasRowsMax || t_lo < 0 || t_hi > kCasSlotsMax || d0 < -127 || d0 > 127)
        return fail(IDF_ESTATE, "internal: cascade schedule of layer %d out of range", l);
    L.cnt = (signed char)cnt; L.rho = (signed char)rho;
    L.t_lo = (signed char)t_lo; L.t_fin = (signed char)t_fin; L.t_hi = (signed char)t_hi;
    L.slot0 = (signed char)(((o_base % g.k_h) + g.k_h) % g.k_h);
    L.d0 = (signed char)d0;
    L.at_start = y0 == 0;
    for (int j = 0; j < cnt && j < kCasRowsMax; ++j) {
        int t = 0;
        const int64_t v = y0 + j + g.p_h, par = g.s_h - 1, sh = g.s_h - 1;      // stride 1 or 2: u % s = u & par, u / s = u >> sh
        for (int ky = 0; ky < g.k_h; ++ky) {
            const int64_t u = v - ky;
            if (u < 0 || (u & par) != 0) continue;
            if (g.h_out > 0 && (u >> sh) >= g.h_out) continue;
            ++t;
        }
        L.taps4[j >> 1] |= (unsigned char)(t << ((j & 1) * 4));
    }
    return IDF_OK;
}

// How a stage whose first layer is l0 takes the segments of a launch: consecutive segments
// together while their rows fit one step (stage 0 gathers the rows of several pushed segments
// itself: those must bring the same number of rows each).  first[m] = first segment of step m.
int cascade_steps_of(const idf_streams::CasGroup &g, int l0, bool merge, int first[kCasSegMax + 1])
{
    int m = 0, q = 0;
    while (q < g.n) {
        int rows = g.seg[q].cnt[l0], e = q + 1;
        while (merge && e < g.n && rows + g.seg[e].cnt[l0] <= kCasRowsMax &&
               (l0 > 0 || g.seg[e].n_rows == g.seg[q].n_rows))
            rows += g.seg[e++].cnt[l0];
        first[m++] = q;
        q = e;
    }
    first[m] = g.n;
    return m;
}

// One launch: stage 0 takes the new segments (none: the stages only move on), stage k those of
// the launch k launches earlier.  staged == false: all layers in one stage, nothing may be on its way.
int cascade_launch(idf_streams *s, const StreamSel &sel, const idf_streams::CasGroup *fresh, bool staged)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    CascadeArgs a{};
    a.n_layers = n;
    a.n_stages = staged ? s->cas_stages : 1;
    for (int k = 0; k <= kCasMaxStages; ++k) a.stage_lo[k] = staged ? s->cas_lo[k] : (k == 0 ? 0 : n);
    a.transit_wr = s->cas_parity;
    for (int l = 0; l < n; ++l) a.layer[l] = s->cas_layer[l];
    for (int k = 0; k < a.n_stages; ++k) {
        const idf_streams::CasGroup *src = k == 0 ? fresh : (s->hist(k - 1).n > 0 ? &s->hist(k - 1) : nullptr);
        if (!src) continue;
        const int l0 = a.stage_lo[k], l1 = a.stage_lo[k + 1];
        int first[kCasSegMax + 1];
        const int n_steps = cascade_steps_of(*src, l0, src->n > 1, first);
        if (n_steps > kCasStepMax) return fail(IDF_ESTATE, "internal: %d steps in one cascade launch", n_steps);
        a.stage_steps[k] = n_steps;
        a.steps_max = std::max(a.steps_max, n_steps);
        int in_rows = 0, out_rows = 0;                  // rows of the launch before this step: into the stage, out of it
        for (int m = 0; m < n_steps; ++m) {
            const int q0 = first[m], q1 = first[m + 1];
            int64_t y0 = 0, cnt = 0;
            for (int q = q0; q < q1; ++q) {
                if (cnt == 0) y0 = src->seg[q].y0[l0];          // (where a segment brings the layer no row, its y0 says nothing)
                cnt += src->seg[q].cnt[l0];
            }
            for (int l = l0; l < l1; ++l) {
                CascadeStep &st = a.step[m][l];
                int rc = cascade_step(net, l, y0, cnt, st);
                if (rc != IDF_OK) return rc;
                if (l == l0) { st.in_off = (short)in_rows; st.seg0 = (signed char)q0; st.seg_rows = (signed char)src->seg[q0].n_rows; }
                if (l == l1 - 1) st.out_off = (short)out_rows;
                const int64_t o_lo = cnt > 0 ? rows_final(net.g[l], y0) : y0, o_fin = cnt > 0 ? rows_final(net.g[l], y0 + cnt) : y0;
                if (cnt <= 0) break;
                y0 = o_lo; cnt = o_fin - o_lo;
            }
            for (int q = q0; q < q1; ++q) { in_rows += src->seg[q].cnt[l0]; out_rows += src->seg[q].cnt[l1]; }
            if (k == a.n_stages - 1) a.out_slot0[m] = src->seg[q0].out_slot0;
        }
    }
    for (int q = 0; fresh && q < fresh->n; ++q) {
        a.in[q] = fresh->seg[q].dev_rows;
        a.in_stream_stride[q] = fresh->seg[q].n_rows * net.in_c;
    }
    a.transit = s->ws + s->cas_transit_off;
    a.transit_stream_stride = (int64_t)kCasSegMax * s->cas_transit_stride;
    a.transit_buf_stride = a.transit_stream_stride * s->B;
    a.out = s->ws + s->out_off; a.out_stride = s->out_stride; a.out_cap = s->out_cap;
    a.stats = (unsigned long long *)(s->ws + s->stats_off);
    a.issued = s->count_issued ? (unsigned long long *)(s->ws + s->issued_off) : nullptr;
    hipError_t e = launch_cascade1d(a, sel, launch_ctx(s, kKindCascade1d, fresh ? fresh->bytes : 0.0));
    if (e != hipSuccess) return dev_fail(e, "cascade launch");
    if (staged) {
        // every launch on its way is one launch older now; the new one takes the place of the oldest
        s->cas_head = (s->cas_head + kCasMaxStages - 1) % kCasMaxStages;
        if (fresh) s->hist(0).take(*fresh); else s->hist(0).n = 0;
        for (int k = s->cas_stages - 1; k < kCasMaxStages; ++k) s->hist(k).n = 0;   // left the last stage
        s->cas_parity ^= 1;
    }
    return IDF_OK;
}

// Segments held back (pushes in step, idf_set_push_batching) get their launch.
int cascade_flush(idf_streams *s)
{
    if (s->cas_pending.n == 0) return IDF_OK;
    StreamSel all{};
    all.n = s->B; all.base = 0; all.pos0 = 0;
    int rc = cascade_launch(s, all, &s->cas_pending, s->cas_stages > 1);
    s->cas_pending.n = 0; s->cas_pending.bytes = 0;
    return rc;
}

// Runs the segments still held back or on their way through the remaining stages.
int cascade_drain(idf_streams *s)
{
    if (!s->use_cascade1d) return IDF_OK;
    int rc = cascade_flush(s);
    if (rc != IDF_OK) return rc;
    StreamSel all{};
    all.n = s->B; all.base = 0; all.pos0 = 0;
    for (;;) {
        bool pending = false;
        for (int k = 0; k < kCasMaxStages - 1; ++k) pending |= s->hist(k).n > 0;
        if (!pending) return IDF_OK;
        rc = cascade_launch(s, all, nullptr, true);
        if (rc != IDF_OK) return rc;
    }
}

// Enqueue everything one group of streams (all at row r, n new rows) needs.
int enqueue_cascade1d(idf_streams *s, const StreamSel &sel, const void *dev_rows, int n_rows, int64_t r,
                      int64_t out_slot0)
{
    // All streams in step: the segment joins those of its launch (stages hold segments of all streams
    // together; held-back segments are segments of all streams).  Any other push first lets everything
    // finish and then runs through all layers at once.
    const bool in_step = sel.base == 0 && sel.pos0 == 0 && sel.n == s->B && (s->cas_stages > 1 || s->cas_batch > 1);
    if (!in_step) {
        int rc = cascade_drain(s);
        if (rc != IDF_OK) return rc;
        idf_streams::CasGroup g;
        g.n = 1;
        cascade_propagate(s, n_rows, r, sel.n, g.seg[0], g.bytes);
        g.seg[0].out_slot0 = out_slot0; g.seg[0].dev_rows = dev_rows; g.seg[0].n_rows = n_rows;
        return cascade_launch(s, sel, &g, false);
    }
    idf_streams::CasGroup &p = s->cas_pending;
    idf_streams::CasSeg &seg = p.seg[p.n];
    cascade_propagate(s, n_rows, r, sel.n, seg, p.bytes);
    seg.out_slot0 = out_slot0; seg.dev_rows = dev_rows; seg.n_rows = n_rows;
    ++p.n;
    // the launch is due when enough segments are held back, or when one more could need more steps
    // than a stage runs in one launch (every stage merges at least as well as the one that merges nothing)
    if (p.n >= s->cas_batch || p.n >= kCasSegMax) return cascade_flush(s);
    int first[kCasSegMax + 1], worst = 0;
    for (int l = 0; l < (int)s->net->g.size(); ++l) worst = std::max(worst, cascade_steps_of(p, l, true, first));
    return worst >= kCasStepMax ? cascade_flush(s) : IDF_OK;
}

// The matrix-core step of conv layer l (with the pool fused behind it, if any) for input row y:
// everything but where the input row lies and where emitted rows go.  rows_out[ky] = index, in
// the layer whose rows leave the step, of the row tap ky emits, or -1.
void make_mfma_step(idf_streams *s, int l, int64_t y, int n_streams, MfmaStep &a, int64_t rows_out[3], double &bytes)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    const int eb = ev_bytes(net.precision);
    const Geom &g = net.g[l];
    const bool pool = l + 1 < n && s->mfma[l + 1] == 2;
    const int lp = pool ? l + 1 : l;
    const bool last_out = lp == n - 1;
    const Geom &gp = net.g[lp];
    a = MfmaStep{};
    a.w = g.w_out; a.c_in = g.c_in; a.c_out = g.c_out; a.c_out_pad = (g.c_out + 63) / 64 * 64;
    a.c_in_rcp = (unsigned)((0x100000000ull + g.c_in - 1) / g.c_in);
    {
        const int chunks = g.c_in / conv3x3_mfma_vl(net.precision);
        a.chunks_rcp = chunks > 1 ? (unsigned)((0x100000000ull + chunks - 1) / chunks) : 0u;
    }
    a.act = g.act; a.shr = g.shr; a.clamp_hi = g.clamp_hi;
    a.layer = l; a.pool_layer = pool ? l + 1 : -1; a.n_layers = n;
    a.tile = conv3x3_mfma_tile(g, n_streams);
    const bool part = l == 0 && s->part.on;
    a.x_lo = part ? s->part.x_lo : 0; a.x_hi = part ? s->part.x_hi : g.w_in;
    const bool first_part = !part || s->part.first, last_part = !part || s->part.last;
    a.skip_clear_tiles = !first_part && !last_part;
    const int64_t fin_after = rows_final(g, y + 1);
    int taps_y = 0;
    for (int ky = 0; ky < 3; ++ky) {
        MfmaTap &t = a.t[ky];
        rows_out[ky] = -1;
        const int64_t o = y + 1 - ky;
        t.valid = o >= 0 && o < g.h_out;
        if (!t.valid) continue;
        ++taps_y;
        t.fresh = first_part && std::max<int64_t>(0, o - 1) >= y;     // later segments of the row continue it
        t.ring_slot = (int)(o % 3);
        const bool fin = last_part && o < fin_after;                  // nothing is final before the row is whole
        if (!fin) { t.emit = kEmitNone; continue; }
        int64_t row = o;                                // row index in the leaving layer
        if (!pool) t.emit = kEmitDirect;
        else if (o % 2 == 0) {
            t.emit = kEmitHold;
            t.store_held = (o / 2 < gp.h_out) && !(o + 1 < fin_after);
            continue;
        } else {
            t.emit = (o - 1 >= rows_final(g, y)) ? kEmitPoolReg : kEmitPoolHeld;
            row = o / 2;
            if (row >= gp.h_out) { t.emit = kEmitHold; t.store_held = 0; continue; }
        }
        rows_out[ky] = row;
    }
    a.taps_y = taps_y;
    a.ring = s->ws + s->ring_off[l]; a.ring_stream_stride = s->ring_stride[l];
    a.held = pool ? s->ws + s->held_off[l + 1] : nullptr;
    a.held_stream_stride = pool ? s->held_stride[l + 1] : 0;
    a.dst = last_out ? (void *)(s->ws + s->out_off) : (void *)(s->ws + s->transit_off[lp]);
    a.dst_stream_stride = last_out ? s->out_stride : s->transit_stride[lp];
    a.to_output = last_out;
    a.wfrag = s->ws + s->wm_off[l];
    if (const size_t ev_at = conv3x3_mfma_event_weights(net.precision, g)) {
        // Up to how many events a tile goes the event path, once the caller has switched it on: a first
        // layer of a few channels whenever the list holds them, elsewhere ev_per_step events per K-step
        // that the contraction would take.
        a.w_ev = s->ws + s->wm_off[l] + ev_at;
        const int vl = conv3x3_mfma_vl(net.precision);
        const int steps = (3 * g.c_in + 2 * vl - 1) / (2 * vl);
        // (layers of more than 16 input channels never take it: their share of the weights would crowd
        // the LDS of every workgroup of the launch for tiles too sparse to exist in practice)
        a.ev_limit = s->ev_per_step == 0 || g.c_in > 16 ? 0
                     : g.c_in < vl ? conv3x3_mfma_event_cap() : std::min(conv3x3_mfma_event_cap(), steps * s->ev_per_step);
    }
    a.bias = net.b_img[l].empty() ? nullptr : s->ws + s->b_off[l];
    a.stats = (unsigned long long *)(s->ws + s->stats_off);
    a.issued = s->count_issued ? (unsigned long long *)(s->ws + s->issued_off) : nullptr;
    ConvStep c{};
    c.g = g; c.y0 = y; c.cnt = 1; c.o_lo = rows_final(g, y); c.o_fin = fin_after;
    c.o_hi = std::max(rows_touched(g, y + 1), c.o_fin);
    c.in_by_position = l == 0; c.to_output = !pool && last_out; c.bias = a.bias;
    bytes = conv_step_bytes(net, c, n_streams);
    if (pool) bytes += n_streams * (double)g.w_out * g.c_out * eb;      // the held row, written or read
}

// One launch for all streams: every conv layer that has a row waiting takes one step, layer 0 on
// row j of the pushed segment (j < 0: no new row, the layers only move on).  What a step emits
// waits for the next layer's step in a later launch.
int stg_tick(idf_streams *s, const void *dev_rows, int n_rows, int j, int64_t r, bool pairs = false)
{
    const idf_net &net = *s->net;
    const int nu = (int)s->stg_unit.size();
    StreamSel all{};
    all.n = s->B; all.base = 0; all.pos0 = 0;
    MfmaBatch b{};
    b.tile = s->stg_tile;
    double bytes_total = 0;
    for (int k = nu - 1; k >= 0; --k) {         // deeper first: they take only rows that were there before
        const int l = s->stg_unit[k];
        const Geom &g = net.g[l];
        // the row the unit takes, and with pairs the one after it if that is there too (same sample)
        int64_t y, y2 = -1;
        int slot = 0, slot2 = 0;
        if (k == 0) {
            if (j < 0) continue;
            y = r + j;
            if (pairs && j + 1 < n_rows) y2 = y + 1;
        } else {
            std::deque<idf_streams::StgRow> &f = s->stg_fifo[k];
            if (f.empty()) continue;
            y = f.front().y; slot = f.front().slot;
            f.pop_front();
            if (pairs && !f.empty() && f.front().y == y + 1) { y2 = y + 1; slot2 = f.front().slot; f.pop_front(); }
        }
        MfmaStep a;
        int64_t rows_out[2][3];
        double bytes = 0;
        make_mfma_step(s, l, y, s->B, a, rows_out[0], bytes);
        const int lp = l - 1;                     // the layer whose rows this one reads: conv or fused pool before it
        if (k == 0) {
            a.in = dev_rows; a.in_stream_stride = (int64_t)n_rows * net.in_w * net.in_c; a.in_by_position = 1;
            a.in_row_off = (int64_t)j * g.w_in * g.c_in;
            a.in_row_off2 = (int64_t)(j + 1) * g.w_in * g.c_in;
            if (s->part.on) { a.in_stream_stride = (int64_t)(s->part.x_hi - s->part.x_lo) * net.in_c; a.in_row_off = -(int64_t)s->part.x_lo * net.in_c; }
        } else {
            a.in = s->ws + s->transit_off[lp]; a.in_stream_stride = s->transit_stride[lp]; a.in_by_position = 0;
            a.in_row_off = (int64_t)slot * g.w_in * g.c_in;
            a.in_row_off2 = (int64_t)slot2 * g.w_in * g.c_in;
        }
        if (y2 >= 0) {
            // The second row's step, folded into the first: rows y and y+1 of c stay in the accumulators in between,
            // and a pool pair that the two rows complete between them keeps its even row in registers.
            MfmaStep a2;
            double bytes2 = 0;
            make_mfma_step(s, l, y2, s->B, a2, rows_out[1], bytes2);
            a.dbl = 1; a.taps_y2 = a2.taps_y;
            for (int ky = 0; ky < 3; ++ky) a.t2[ky] = a2.t[ky];
            for (int ky = 0; ky < 2; ++ky)
                if (a.t[ky].valid && a.t[ky].emit == kEmitNone) a.t[ky].emit = kEmitKeep;
            if (a.t[2].valid && a.t[2].emit == kEmitHold && a.t2[2].valid && a.t2[2].emit == kEmitPoolHeld) {
                a.t[2].store_held = 0; a.t2[2].emit = kEmitPoolReg;
            }
            // what the pair has to move by the method: the two rows of c between the two input rows neither leave
            // the chip nor come back (two rows written and two read fewer than two steps)
            bytes += bytes2 - (double)s->B * 4.0 * g.w_out * g.c_out * 4.0;
        }
        for (int sub = 0; sub < (y2 >= 0 ? 2 : 1); ++sub) {
            MfmaTap *t = sub ? a.t2 : a.t;
            for (int ky = 2; ky >= 0; --ky) {     // increasing row index
                if (rows_out[sub][ky] < 0) continue;
                if (k == nu - 1) {
                    t[ky].dst_slot = s->stg_out_next;
                    s->stg_out_next = (s->stg_out_next + 1) % s->out_cap;
                } else {
                    const int wslot = (int)(s->stg_seq[k]++ % s->stg_slots);
                    t[ky].dst_slot = wslot;
                    s->stg_fifo[k + 1].push_back({rows_out[sub][ky], wslot});
                }
            }
        }
        b.st[b.n++] = a;
        bytes_total += bytes;
    }
    if (b.n == 0) return IDF_OK;
    // Dispatch order of the steps within the launch: deepest layer first (its workgroups run longest).
    // When the launch holds more workgroups than the chip takes at once, the others follow shallowest
    // first: the short workgroups of the first layers then finish early and hand their places to what
    // did not fit.  (Measured: 4 % faster on the VGG-style workload, whose launches are 1.25 rounds;
    // 15 % slower on the small-image workload, whose launches fit at once: hence the condition.)
    if (b.n >= 3 && s->cus > 0) {
        long wgs = 0;
        for (int k = 0; k < b.n; ++k) wgs += (long)conv3x3_mfma_tiles(b.tile, b.st[k].w, b.st[k].c_out) * s->B;
        if (wgs > (long)s->cus * conv3x3_mfma_batch_resident(net.precision, b.tile)) std::reverse(b.st + 1, b.st + b.n);
    }
    hipError_t e = launch_conv3x3_mfma_batch(net.precision, b, all, launch_ctx(s, kKindConvMfma, bytes_total, -1));
    return e == hipSuccess ? IDF_OK : dev_fail(e, "staged mfma conv launch");
}

bool stg_pending(const idf_streams *s, size_t more_than)
{
    for (const auto &f : s->stg_fifo) if (f.size() > more_than) return true;
    return false;
}

int stg_drain(idf_streams *s)
{
    while (s->stg2d && stg_pending(s, 0)) {
        int rc = stg_tick(s, nullptr, 0, -1, 0);
        if (rc != IDF_OK) return rc;
    }
    return IDF_OK;
}

// Everything still between stages or layers is enqueued: afterwards the work in the stream is
// that of every pushed row having gone through every layer it can influence.
int pipeline_drain(idf_streams *s)
{
    int rc = cascade_drain(s);
    return rc != IDF_OK ? rc : stg_drain(s);
}

int enqueue_cascade(idf_streams *s, const StreamSel &sel, const void *dev_rows, int n_rows, int64_t r,
                    int64_t out_slot0)
{
    if (s->use_cascade1d) return enqueue_cascade1d(s, sel, dev_rows, n_rows, r, out_slot0);
    if (s->stg2d) {
        if (sel.base == 0 && sel.pos0 == 0 && sel.n == s->B) {
            if (!stg_pending(s, 0)) s->stg_out_next = out_slot0;
            // A push of several rows goes through two rows per launch (every unit that finds two rows waiting takes both
            // in one step); a push of one row, and the ticks that only move the layers on, take one.
            const bool pairs = s->stg_pairs && !s->part.on && s->ev_per_step == 0;
            for (int j = 0; j < n_rows;) {
                const bool two = pairs && j + 1 < n_rows;
                int rc = stg_tick(s, dev_rows, n_rows, j, r, two);
                // the hand-over rings hold kStgSlots rows: never let more than kStgWait wait
                while (rc == IDF_OK && stg_pending(s, kStgWait)) rc = stg_tick(s, nullptr, 0, -1, 0);
                if (rc != IDF_OK) return rc;
                j += two ? 2 : 1;
            }
            return IDF_OK;
        }
        int rc = stg_drain(s);                     // some streams only: finish what is on its way, then layer by layer
        if (rc != IDF_OK) return rc;
    }
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    const int eb = ev_bytes(net.precision);
    unsigned long long *stats = (unsigned long long *)(s->ws + s->stats_off);
    const void *in = dev_rows;
    int64_t in_stride = (int64_t)n_rows * net.in_w * net.in_c;
    int64_t in_row0 = r;
    int by_pos = 1;
    int64_t y0 = r;
    int64_t cnt = n_rows;
    for (int l = 0; l < n && cnt > 0; ++l) {
        const Geom &g = net.g[l];
        const bool last = l == n - 1;
        const int64_t o_lo = rows_final(g, y0), o_fin = rows_final(g, y0 + cnt);
        void *dst = last ? (void *)(s->ws + s->out_off) : (void *)(s->ws + s->transit_off[l]);
        const int64_t dst_stride = last ? s->out_stride : s->transit_stride[l];
        if (!last && o_fin - o_lo > s->transit_cap[l])
            return fail(IDF_ESTATE, "internal: layer %d would emit %lld rows, room for %d", l,
                        (long long)(o_fin - o_lo), s->transit_cap[l]);
        if (g.kind == IDF_CONV && s->mfma[l] == 1) {
            // one launch per arriving row; a pool that follows is done in the epilogue
            const bool pool = l + 1 < n && s->mfma[l + 1] == 2;
            const int lp = pool ? l + 1 : l;                        // layer whose rows leave this step
            const bool last_out = lp == n - 1;
            const Geom &gp = net.g[lp];
            const int64_t e_lo = pool ? rows_final(gp, o_lo) : o_lo, e_fin = pool ? rows_final(gp, o_fin) : o_fin;
            void *edst = last_out ? (void *)(s->ws + s->out_off) : (void *)(s->ws + s->transit_off[lp]);
            const int64_t edst_stride = last_out ? s->out_stride : s->transit_stride[lp];
            if (!last_out && e_fin - e_lo > s->transit_cap[lp])
                return fail(IDF_ESTATE, "internal: layer %d would emit %lld rows, room for %d", lp,
                            (long long)(e_fin - e_lo), s->transit_cap[lp]);
            for (int64_t y = y0; y < y0 + cnt; ++y) {
                MfmaStep a;
                int64_t rows_out[3];
                double bytes = 0;
                make_mfma_step(s, l, y, sel.n, a, rows_out, bytes);
                for (int ky = 0; ky < 3; ++ky) {
                    if (rows_out[ky] < 0) continue;
                    a.t[ky].dst_slot = rows_out[ky] - e_lo;
                    if (last_out) a.t[ky].dst_slot = (out_slot0 + a.t[ky].dst_slot) % s->out_cap;
                }
                a.in = in; a.in_stream_stride = in_stride; a.in_by_position = by_pos;
                a.in_row_off = (y - in_row0) * (int64_t)g.w_in * g.c_in;
                if (l == 0 && s->part.on) { a.in_stream_stride = (int64_t)(s->part.x_hi - s->part.x_lo) * net.in_c; a.in_row_off = -(int64_t)s->part.x_lo * net.in_c; }
                hipError_t e = launch_conv3x3_mfma(net.precision, a, sel, launch_ctx(s, kKindConvMfma, bytes, l));
                if (e != hipSuccess) return dev_fail(e, "mfma conv launch");
            }
            in = edst; in_stride = edst_stride; in_row0 = e_lo; by_pos = 0;
            y0 = e_lo; cnt = e_fin - e_lo;
            if (pool) ++l;
            continue;
        } else if (g.kind == IDF_CONV) {
            const int max_rows = conv_generic_max_rows(g.c_out);
            int64_t yy = y0;
            while (yy < y0 + cnt) {
                int64_t c = y0 + cnt - yy;
                auto touched = [&](int64_t cc) {
                    return std::max(rows_touched(g, yy + cc), rows_final(g, yy + cc)) - rows_final(g, yy);
                };
                while (c > 1 && touched(c) > max_rows) c = (c + 1) / 2;
                ConvStep a{};
                a.g = g; a.layer = l; a.y0 = yy; a.cnt = (int)c;
                a.o_lo = rows_final(g, yy); a.o_fin = rows_final(g, yy + c);
                a.o_hi = std::max(rows_touched(g, yy + c), a.o_fin);
                a.ring_rows = g.k_h;
                a.in = in; a.in_stream_stride = in_stride; a.in_row0 = in_row0; a.in_by_position = by_pos;
                a.ring = s->ws + s->ring_off[l]; a.ring_stream_stride = s->ring_stride[l];
                a.dst = dst; a.dst_stream_stride = dst_stride; a.dst_row0 = o_lo; a.dst_slot0 = out_slot0;
                a.to_output = last; a.out_cap = s->out_cap;
                a.w = s->ws + s->w_off[l];
                a.bias = net.b_img[l].empty() ? nullptr : s->ws + s->b_off[l];
                a.stats = stats; a.n_layers = n;
                if (l == 0 && s->part.on) {       // the pixel segment that completes a row (c == 1): layer 0 takes only its columns
                    a.x_lo = s->part.x_lo; a.x_hi = s->part.x_hi; a.cont = !s->part.first;
                    a.in_stream_stride = (int64_t)(s->part.x_hi - s->part.x_lo) * net.in_c;
                }
                conv_generic_plan(a);
                hipError_t e = launch_conv_generic(net.precision, a, sel,
                                                   launch_ctx(s, kKindConvGeneric, conv_step_bytes(net, a, sel.n), l));
                if (e != hipSuccess) return dev_fail(e, "conv launch");
                yy += c;
            }
        } else {
            PoolStep a{};
            a.g = g; a.layer = l; a.y0 = y0; a.cnt = (int)cnt; a.o_lo = o_lo; a.o_fin = o_fin;
            const int64_t y_last = y0 + cnt - 1;
            a.hold_new = (y_last % 2 == 0) && (g.h_out == 0 || y_last / 2 < g.h_out);
            a.in = in; a.in_stream_stride = in_stride; a.in_row0 = in_row0; a.in_by_position = by_pos;
            a.held = s->ws + s->held_off[l]; a.held_stream_stride = s->held_stride[l];
            a.dst = dst; a.dst_stream_stride = dst_stride; a.dst_row0 = o_lo; a.dst_slot0 = out_slot0;
            a.to_output = last; a.out_cap = s->out_cap;
            a.stats = stats; a.n_layers = n;
            const double row_in = (double)g.w_in * g.c_out * eb, row_out = (double)g.w_out * g.c_out;
            const double bytes = sel.n * (cnt * row_in + (a.hold_new ? row_in : 0) + (y0 % 2 ? row_in : 0) +
                                          (double)(o_fin - o_lo) * row_out * (last ? 4 : eb));
            hipError_t e = launch_pool_generic(net.precision, a, sel, launch_ctx(s, kKindPoolGeneric, bytes, l));
            if (e != hipSuccess) return dev_fail(e, "pool launch");
        }
        in = dst; in_stride = dst_stride; in_row0 = o_lo; by_pos = 0;
        y0 = o_lo; cnt = o_fin - o_lo;
    }
    return IDF_OK;
}

// One stream's pieces of the workspace, in the order they are laid out in a snapshot.
template <class F> void for_each_state_piece(const idf_streams *s, int id, F &&f)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    const int eb = ev_bytes(net.precision);
    for (int l = 0; l < n; ++l) {
        if (net.g[l].kind == IDF_CONV) f(s->ring_off[l] + (size_t)id * s->ring_stride[l] * 4, (size_t)s->ring_stride[l] * 4);
        else f(s->held_off[l] + (size_t)id * s->held_stride[l] * eb, (size_t)s->held_stride[l] * eb);
    }
    f(s->stats_off + (size_t)id * n * 2 * sizeof(unsigned long long), (size_t)n * 2 * sizeof(unsigned long long));
    f(s->issued_off + (size_t)id * n * sizeof(unsigned long long), (size_t)n * sizeof(unsigned long long));
    f(s->head_off + (size_t)id * net.out_c * sizeof(double), (size_t)net.out_c * sizeof(double));
}
// The band of rows of every level that the input rows [a, b) reach: lo[lv], hi[lv] for lv = 0 ..
// n_layers (level 0 is the input itself).  With `everything` every row of every level.
void eager_bands(const idf_net &net, int64_t a, int64_t b, bool everything, std::vector<int64_t> &lo, std::vector<int64_t> &hi)
{
    const int n = (int)net.g.size();
    lo.assign(n + 1, 0); hi.assign(n + 1, 0);
    lo[0] = a; hi[0] = b;
    for (int l = 0; l < n; ++l) {
        const Geom &g = net.g[l];
        int64_t oa = 0, ob = 0;
        if (b > a) {
            if (g.kind == IDF_CONV) {
                // output rows whose footprint meets [a, b)
                const int64_t t = a + g.p_h - g.k_h + 1;
                oa = t <= 0 ? 0 : (t + g.s_h - 1) / g.s_h;
                ob = std::min<int64_t>(g.h_out, (b - 1 + g.p_h) / g.s_h + 1);
            } else {
                oa = a / 2; ob = std::min<int64_t>(g.h_out, (b - 1) / 2 + 1);
            }
            if (ob < oa) ob = oa;
        }
        if (everything) { oa = 0; ob = g.h_out; }
        lo[l + 1] = oa; hi[l + 1] = ob;
        a = oa; b = ob;
    }
}

// Layout of the eager-emission workspace for B streams pushed at most max_seg rows at a time;
// returns its size.  Nets without biases keep, per level, a ring of the rows a push can reach plus
// those a pool still looks at (every other row is final and forgotten, or still all zero); the
// last level's announced values -- the output -- are kept whole.  With biases every neuron of the
// net announces a value before any input arrives, so every level is kept whole.
size_t eager_layout(const idf_net &net, int B, int max_seg, idf_streams::Eager *e)
{
    const int n = (int)net.g.size();
    bool ring = true;
    for (int l = 0; l < n; ++l) ring = ring && net.b_img[l].empty();
    std::vector<int64_t> row_elems(n + 1);
    std::vector<int> rows(n + 1), ann_rows(n + 1), cd_rows(n + 1);
    row_elems[0] = (int64_t)net.in_w * net.in_c; rows[0] = net.in_h;
    for (int l = 0; l < n; ++l) { row_elems[l + 1] = (int64_t)net.g[l].w_out * net.g[l].c_out; rows[l + 1] = net.g[l].h_out; }
    for (int lv = 0; lv <= n; ++lv) ann_rows[lv] = cd_rows[lv] = rows[lv];
    if (ring) {
        std::vector<int64_t> need(n + 1, 1), lo, hi;
        for (int64_t a = 0; a < net.in_h; ++a) {
            eager_bands(net, a, std::min<int64_t>(a + max_seg, net.in_h), false, lo, hi);
            for (int lv = 0; lv <= n; ++lv) {
                int64_t first = lo[lv];
                // a pool re-evaluates whole windows: it also looks at the row before its band begins
                if (lv < n && net.g[lv].kind == IDF_MAXPOOL && hi[lv + 1] > lo[lv + 1]) first = std::min(first, 2 * lo[lv + 1]);
                need[lv] = std::max(need[lv], hi[lv] - first);
            }
        }
        for (int lv = 0; lv <= n; ++lv) {
            cd_rows[lv] = (int)std::min<int64_t>(rows[lv], need[lv]);
            ann_rows[lv] = lv == n ? rows[lv] : cd_rows[lv];
        }
    }
    size_t off = 0;
    std::vector<size_t> ann(n + 1), c(n + 1, 0), dlt(n + 1);
    for (int lv = 0; lv <= n; ++lv) {
        ann[lv] = off; off = align_up(off + (size_t)ann_rows[lv] * row_elems[lv] * 4 * B);
        dlt[lv] = off; off = align_up(off + (size_t)cd_rows[lv] * row_elems[lv] * 4 * B);
        if (lv > 0 && net.g[lv - 1].kind == IDF_CONV) { c[lv] = off; off = align_up(off + (size_t)cd_rows[lv] * row_elems[lv] * 4 * B); }
    }
    if (e) {
        e->ring = ring; e->row_elems = row_elems; e->rows = rows; e->ann_rows = ann_rows; e->cd_rows = cd_rows;
        e->ann_off = ann; e->c_off = c; e->dlt_off = dlt;
    }
    return off;
}

// One pass of eager emission for a selection of streams: the input rows [a, b) (pushed rows, or
// none when only the biases announce themselves) and, layer by layer, the band of rows they reach.
int eager_pass(idf_streams *s, const StreamSel &sel, const void *dev_rows, int n_rows, int64_t a, int64_t b, bool init_bias)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    idf_streams::Eager &E = s->eager;
    unsigned long long *stats = (unsigned long long *)(s->ws + s->stats_off);
    std::vector<int64_t> lo, hi, seen_lo, seen_hi;
    eager_bands(net, a, b, init_bias, lo, hi);
    eager_bands(net, 0, a, false, seen_lo, seen_hi);          // seen_hi[lv]: rows of level lv reached before this pass
    const int round_bf16 = net.precision == IDF_PREC_BF16;
    auto fresh_from = [&](int lv) { return E.ring ? (int)seen_hi[lv] : (int)E.rows[lv]; };    // whole maps are cleared when a sample begins
    if (dev_rows) {
        EagerStep st{};
        st.layer = 0; st.n_layers = n; st.o_lo = (int)a; st.o_hi = (int)b; st.w_out = net.in_w; st.c_out = net.in_c;
        st.in = dev_rows; st.in_stream_stride = (int64_t)n_rows * net.in_w * net.in_c;
        st.ann = E.ws + E.ann_off[0]; st.dlt_out = E.ws + E.dlt_off[0];
        st.ann_rows = E.ann_rows[0]; st.dlt_rows = E.cd_rows[0];
        st.ann_stride = (int64_t)E.ann_rows[0] * E.row_elems[0]; st.dlt_stride = (int64_t)E.cd_rows[0] * E.row_elems[0];
        st.fresh_lo = fresh_from(0);
        st.stats = stats;
        hipError_t e = launch_eager(net.precision, 0, st, sel,
                                    launch_ctx(s, kKindEager, (double)(b - a) * net.in_w * net.in_c * sel.n * 9.0, 0));
        if (e != hipSuccess) return dev_fail(e, "eager input launch");
    }
    for (int l = 0; l < n && hi[l] > lo[l]; ++l) {
        const Geom &g = net.g[l];
        if (hi[l + 1] <= lo[l + 1]) break;
        EagerStep st{};
        st.g = g; st.layer = l; st.n_layers = n; st.i_lo = (int)lo[l]; st.i_hi = (int)hi[l]; st.init_bias = init_bias;
        st.o_lo = (int)lo[l + 1]; st.o_hi = (int)hi[l + 1];
        st.fresh_lo = fresh_from(l + 1);
        st.in_hi = E.ring ? (int)hi[l] : (int)E.rows[l];
        st.round_bf16 = round_bf16 && l + 1 < n;              // the last layer's output is not rounded
        st.dlt_in = E.ws + E.dlt_off[l]; st.ann_in = E.ws + E.ann_off[l];
        st.in_rows = E.cd_rows[l];                              // (announced values of a level that feeds a layer are kept as long as its deltas)
        st.in_map_stride = (int64_t)E.cd_rows[l] * E.row_elems[l];
        st.c = g.kind == IDF_CONV ? E.ws + E.c_off[l + 1] : nullptr;
        st.ann = E.ws + E.ann_off[l + 1]; st.dlt_out = E.ws + E.dlt_off[l + 1];
        st.c_rows = st.dlt_rows = E.cd_rows[l + 1]; st.ann_rows = E.ann_rows[l + 1];
        st.c_stride = st.dlt_stride = (int64_t)E.cd_rows[l + 1] * E.row_elems[l + 1];
        st.ann_stride = (int64_t)E.ann_rows[l + 1] * E.row_elems[l + 1];
        st.w = g.kind == IDF_CONV ? s->ws + s->w_off[l] : nullptr;
        st.bias = (g.kind == IDF_CONV && !net.b_img[l].empty()) ? s->ws + s->b_off[l] : nullptr;
        st.stats = stats;
        const double cells = (double)(hi[l + 1] - lo[l + 1]) * g.w_out * g.c_out * sel.n;
        hipError_t e = launch_eager(net.precision, g.kind == IDF_CONV ? 1 : 2, st, sel,
                                    launch_ctx(s, kKindEager, cells * 16.0, l));
        if (e != hipSuccess) return dev_fail(e, "eager layer launch");
    }
    return IDF_OK;
}

int eager_push(idf_streams *s, const int32_t *stream_ids, int n_ids, const void *dev_rows, int n_rows)
{
    const idf_net &net = *s->net;
    const int n = (int)net.g.size();
    idf_streams::Eager &E = s->eager;
    std::map<int64_t, std::vector<std::pair<int, int>>> groups;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        const StreamHost &h = s->h[id];
        if (h.r + n_rows > net.in_h)
            return fail(IDF_ESTATE, "stream %d: rows %lld..%lld run past the sample of %d rows", id, (long long)h.r,
                        (long long)(h.r + n_rows - 1), net.in_h);
        groups[h.r].push_back({i, id});
    }
    bool any_bias = false;
    for (int l = 0; l < n; ++l) any_bias |= !net.b_img[l].empty();
    for (auto &kv : groups) {
        const int64_t r = kv.first;
        if (r == 0) {
            // a sample begins: all state zero (Sec. 3), then the biases announce themselves.  Rings need
            // no clearing (a row starts from zero when it is first reached); what is kept whole does.
            int rc0 = for_each_selection(kv.second, [&](const StreamSel &sel) {
                // streams lie side by side in every map: one fill per map and run of streams
                for (int k = 0; k < (sel.base >= 0 ? 1 : sel.n); ++k) {
                    const int first = sel.base >= 0 ? sel.base : sel.ids[k], cnt = sel.base >= 0 ? sel.n : 1;
                    for (int lv = 0; lv <= n; ++lv) {
                        hipError_t e = hipSuccess;
                        if (!E.ring || lv == n) {
                            const size_t per = (size_t)E.ann_rows[lv] * E.row_elems[lv] * 4;
                            e = launch_fill_zero(E.ws + E.ann_off[lv] + (size_t)first * per, per * cnt, s->st);
                        }
                        if (!E.ring) {
                            const size_t per = (size_t)E.cd_rows[lv] * E.row_elems[lv] * 4, at = (size_t)first * per;
                            if (e == hipSuccess) e = launch_fill_zero(E.ws + E.dlt_off[lv] + at, per * cnt, s->st);
                            if (e == hipSuccess && lv > 0 && net.g[lv - 1].kind == IDF_CONV)
                                e = launch_fill_zero(E.ws + E.c_off[lv] + at, per * cnt, s->st);
                        }
                        if (e != hipSuccess) return dev_fail(e, "eager reset");
                    }
                }
                return (int)IDF_OK;
            });
            if (rc0 != IDF_OK) return rc0;
        }
        int rc = for_each_selection(kv.second, [&](const StreamSel &sel) {
            if (r == 0 && any_bias) {
                int rc2 = eager_pass(s, sel, nullptr, 0, 0, net.in_h, true);
                if (rc2 != IDF_OK) return rc2;
            }
            return eager_pass(s, sel, dev_rows, n_rows, r, r + n_rows, false);
        });
        if (rc != IDF_OK) return rc;
    }
    for (int i = 0; i < n_ids; ++i) {
        StreamHost &h = s->h[stream_ids ? stream_ids[i] : i];
        h.r += n_rows;
        h.eager_rows = h.r;                      // rows of the current sample the levels have seen
        if (h.r == net.in_h) h.r = 0;
    }
    return IDF_OK;
}

// The averaging units take in the output rows completed since they last did.  Must run before
// read_outputs gives those rows' slots free.
int head_catch_up(idf_streams *s, const int32_t *stream_ids, int n_ids)
{
    if (!s->head_on) return IDF_OK;
    const idf_net &net = *s->net;
    struct Key { int64_t slot; int64_t n; int zero; int64_t count; int64_t row0;
                 bool operator<(const Key &o) const { return std::tie(slot, n, zero, count, row0) < std::tie(o.slot, o.n, o.zero, o.count, o.row0); } };
    std::map<Key, std::vector<std::pair<int, int>>> groups;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        StreamHost &h = s->h[id];
        const int64_t b = h.out_written;
        int64_t a = h.head_done;
        if (b <= a) continue;
        int zero = 0;
        if (net.out_h > 0) {
            const int64_t sb = (b - 1) / net.out_h * net.out_h;      // first row of the newest sample with a row
            if (sb > h.head_base) { zero = 1; a = std::max(a, sb); h.head_base = sb; }
        }
        if (b - a > s->out_cap) return fail(IDF_ESTATE, "internal: rows for the averaging units no longer in the output area");
        if (s->head_units && a == h.head_base) zero = 1;      // first rows of a sample: the units start from their bias
        groups[Key{a % s->out_cap, b - a, zero, (b - h.head_base) * (int64_t)net.out_w, a - h.head_base}].push_back({i, id});
        h.head_done = b;
    }
    HeadAcc a{};
    a.src = s->ws + s->out_off; a.src_stream_stride = s->out_stride; a.out_cap = s->out_cap;
    a.w = net.out_w; a.c = net.out_c; a.is_int = net.precision == IDF_PREC_I8;
    a.sums = (double *)(s->ws + s->head_off); a.mean = a.sums + (size_t)s->B * net.out_c;
    for (auto &kv : groups) {
        a.zero_first = kv.first.zero; a.count = (double)kv.first.count;
        const int64_t slot = kv.first.slot;
        const int n = (int)kv.first.n;
        int rc = for_each_selection(kv.second, [&](const StreamSel &sel) {
            hipError_t e = launch_head_accumulate(a, sel, slot, n,
                                                  launch_ctx(s, kKindHead, 4.0 * n * net.out_w * net.out_c * sel.n));
            if (e == hipSuccess && s->head_units) {
                HeadUnits u{};
                u.src = a.src; u.src_stream_stride = a.src_stream_stride; u.out_cap = a.out_cap; u.w = a.w; u.c = a.c;
                u.n_units = s->head_units; u.is_int = a.is_int; u.zero_first = kv.first.zero; u.row0 = kv.first.row0;
                u.map_elems = (int64_t)net.out_h * net.out_w * net.out_c;
                u.weights = (const float *)s->head_units_ws;
                u.bias = s->head_units_bias ? u.weights + (size_t)s->head_units * u.map_elems : nullptr;
                u.values = (double *)(s->head_units_ws + align_up(((size_t)s->head_units * u.map_elems + s->head_units) * 4));
                e = launch_head_units(u, sel, slot, n, launch_ctx(s, kKindHead, 8.0 * n * net.out_w * net.out_c * sel.n * s->head_units));
            }
            return e == hipSuccess ? IDF_OK : dev_fail(e, "head launch");
        });
        if (rc != IDF_OK) return rc;
    }
    return IDF_OK;
}

int open_on(idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows, const Layout &L, void *dev_workspace,
            size_t workspace_bytes, void *hip_stream, idf_streams **out);

}  // namespace

// -----------------------------------------------------------------------------------------
extern "C" {

const char *idf_last_error(void) { return g_err.c_str(); }

int idf_create_net(const idf_net_desc *d, const void *const *weights, const void *const *biases,
                   idf_net **out)
{
    if (!d || !out || !d->layers) return fail(IDF_EINVAL, "null argument");
    *out = nullptr;
    if (d->precision < IDF_PREC_F32 || d->precision > IDF_PREC_I8) return fail(IDF_EINVAL, "unknown precision %d", d->precision);
    if (d->n_layers < 1 || d->n_layers > kMaxLayers) return fail(IDF_EINVAL, "n_layers %d outside [1, %d]", d->n_layers, kMaxLayers);
    if (d->in_h < 0 || d->in_w < 1 || d->in_c < 1) return fail(IDF_EINVAL, "bad input shape %d x %d x %d", d->in_h, d->in_w, d->in_c);
    idf_net *net = new (std::nothrow) idf_net;
    if (!net) return fail(IDF_ENOMEM, "out of host memory");
    net->precision = d->precision; net->in_h = d->in_h; net->in_w = d->in_w; net->in_c = d->in_c;
    int h = d->in_h, w = d->in_w, c = d->in_c;
    int rc = IDF_OK;
    for (int l = 0; l < d->n_layers && rc == IDF_OK; ++l) {
        const idf_layer &L = d->layers[l];
        Geom g{};
        g.kind = L.kind; g.c_in = L.c_in; g.c_out = L.c_out; g.k_h = L.k_h; g.k_w = L.k_w;
        g.s_h = L.s_h; g.s_w = L.s_w; g.p_h = L.p_h; g.p_w = L.p_w; g.act = L.act; g.shr = L.shr; g.clamp_hi = L.clamp_hi;
        g.h_in = h; g.w_in = w;
        if (L.kind != IDF_CONV && L.kind != IDF_MAXPOOL) rc = fail(IDF_EINVAL, "layer %d: unknown kind %d", l, L.kind);
        else if (L.c_in != c || L.c_out < 1) rc = fail(IDF_EINVAL, "layer %d: c_in %d does not follow %d channels", l, L.c_in, c);
        else if (L.k_h < 1 || L.k_w < 1 || L.s_h < 1 || L.s_w < 1 || L.p_h < 0 || L.p_w < 0) rc = fail(IDF_EINVAL, "layer %d: bad kernel/stride/padding", l);
        else if (d->in_h == 0 && L.p_h != 0) rc = fail(IDF_EINVAL, "layer %d: row padding on an unbounded stream", l);
        else if (L.kind == IDF_MAXPOOL && !(L.c_out == L.c_in && L.k_h == 2 && L.s_h == 2 && L.p_h == 0 && L.p_w == 0 &&
                                            ((L.k_w == 2 && L.s_w == 2) || (L.k_w == 1 && L.s_w == 1))))
            rc = fail(IDF_EINVAL, "layer %d: pool must be 2 x {1,2}, stride = window, no padding", l);
        else if (L.kind == IDF_CONV && (L.act < IDF_ACT_NONE || L.act > IDF_ACT_RELU_SHR_CLAMP)) rc = fail(IDF_EINVAL, "layer %d: unknown activation", l);
        else if (L.kind == IDF_CONV && (!weights || !weights[l])) rc = fail(IDF_EINVAL, "layer %d: no weights", l);
        if (rc != IDF_OK) break;
        g.h_out = d->in_h ? out_size(h, L.k_h, L.s_h, L.p_h) : 0;
        g.w_out = out_size(w, L.k_w, L.s_w, L.p_w);
        if ((d->in_h && g.h_out < 1) || g.w_out < 1) { rc = fail(IDF_EINVAL, "layer %d: window larger than its input", l); break; }
        const bool last = l == d->n_layers - 1;
        if (L.kind == IDF_CONV) {
            if (L.act == IDF_ACT_RELU_SHR_CLAMP && d->precision != IDF_PREC_I8) { rc = fail(IDF_EUNSUPPORTED, "layer %d: shift/clamp activation needs int8 precision", l); break; }
            if (L.act == IDF_ACT_RELU_SHR_CLAMP && (L.shr < 0 || L.shr > 30 || L.clamp_hi < 0 || L.clamp_hi > 127)) { rc = fail(IDF_EINVAL, "layer %d: shr/clamp_hi out of range", l); break; }
            if (d->precision == IDF_PREC_I8 && !last && L.act != IDF_ACT_RELU_SHR_CLAMP) { rc = fail(IDF_EUNSUPPORTED, "layer %d: int8 events between layers need the shift/clamp activation", l); break; }
            if (L.k_h > conv_generic_max_rows(L.c_out)) { rc = fail(IDF_EUNSUPPORTED, "layer %d: kernel height %d too large", l, L.k_h); break; }
        } else if (last && d->precision != IDF_PREC_F32) { rc = fail(IDF_EUNSUPPORTED, "a pool as the last layer needs float32 precision"); break; }
        net->g.push_back(g);
        net->w_img.emplace_back(); net->b_img.emplace_back(); net->wm_img.emplace_back();
        if (L.kind == IDF_CONV) {
            const int wb = w_bytes(d->precision);
            std::vector<unsigned char> &img = net->w_img.back();
            img.resize((size_t)L.k_h * L.k_w * L.c_in * L.c_out * wb);
            const unsigned char *src = (const unsigned char *)weights[l];
            for (int co = 0; co < L.c_out; ++co)
            for (int ci = 0; ci < L.c_in; ++ci)
            for (int ky = 0; ky < L.k_h; ++ky)
            for (int kx = 0; kx < L.k_w; ++kx) {
                size_t s_idx = (((size_t)co * L.c_in + ci) * L.k_h + ky) * L.k_w + kx;
                size_t d_idx = (((size_t)ky * L.k_w + kx) * L.c_in + ci) * L.c_out + co;
                memcpy(&img[d_idx * wb], src + s_idx * wb, wb);
            }
            if (conv3x3_mfma_eligible(d->precision, g)) {
                net->wm_img.back().resize(conv3x3_mfma_pack(d->precision, g, nullptr, nullptr));
                conv3x3_mfma_pack(d->precision, g, img.data(), net->wm_img.back().data());
            }
            if (biases && biases[l]) {
                net->b_img.back().resize((size_t)L.c_out * 4);
                memcpy(net->b_img.back().data(), biases[l], (size_t)L.c_out * 4);
            }
        }
        h = g.h_out; w = g.w_out; c = L.c_out;
    }
    if (rc != IDF_OK) { delete net; return rc; }
    net->out_h = h; net->out_w = w; net->out_c = c;
    *out = net;
    return IDF_OK;
}

int idf_create_net_columnwise(const idf_net_desc *d, const void *const *weights, const void *const *biases,
                              idf_net **out)
{
    if (!d || !out || !d->layers) return fail(IDF_EINVAL, "null argument");
    *out = nullptr;
    if (d->n_layers < 1 || d->n_layers > kMaxLayers) return fail(IDF_EINVAL, "n_layers %d outside [1, %d]", d->n_layers, kMaxLayers);
    if (d->precision < IDF_PREC_F32 || d->precision > IDF_PREC_I8) return fail(IDF_EINVAL, "unknown precision %d", d->precision);
    // The same network with the two image axes exchanged: what streams in is then a column.
    std::vector<idf_layer> lt(d->layers, d->layers + d->n_layers);
    std::vector<std::vector<unsigned char>> wt(d->n_layers);
    std::vector<const void *> wp(d->n_layers, nullptr);
    const size_t wb = (size_t)w_bytes(d->precision);
    for (int l = 0; l < d->n_layers; ++l) {
        idf_layer &L = lt[l];
        std::swap(L.k_h, L.k_w); std::swap(L.s_h, L.s_w); std::swap(L.p_h, L.p_w);
        if (L.kind != IDF_CONV || !weights || !weights[l]) continue;
        if (L.c_in < 1 || L.c_out < 1 || L.k_h < 1 || L.k_w < 1) return fail(IDF_EINVAL, "layer %d: bad shape", l);
        // [c_out][c_in][k_h][k_w] of the image orientation -> the same with the two kernel axes exchanged
        const int kh = L.k_w, kw = L.k_h;                      // of the image orientation
        wt[l].resize((size_t)L.c_out * L.c_in * kh * kw * wb);
        const unsigned char *src = (const unsigned char *)weights[l];
        for (size_t oc = 0; oc < (size_t)L.c_out * L.c_in; ++oc)
            for (int ky = 0; ky < kh; ++ky)
                for (int kx = 0; kx < kw; ++kx)
                    memcpy(&wt[l][((oc * kw + kx) * kh + ky) * wb], src + ((oc * kh + ky) * kw + kx) * wb, wb);
        wp[l] = wt[l].data();
    }
    idf_net_desc t = *d;
    t.in_h = d->in_w; t.in_w = d->in_h; t.layers = lt.data();
    if (t.in_w < 1) return fail(IDF_EINVAL, "column-wise presentation needs the column length in_h");
    return idf_create_net(&t, wp.data(), biases, out);
}

int idf_create_net_volume(const idf_volume_desc *d, const void *const *weights, const void *const *biases, idf_net **out)
{
    if (!d || !out || !d->layers) return fail(IDF_EINVAL, "null argument");
    *out = nullptr;
    if (d->n_layers < 1 || d->n_layers > kMaxLayers) return fail(IDF_EINVAL, "n_layers %d outside [1, %d]", d->n_layers, kMaxLayers);
    if (d->precision < IDF_PREC_F32 || d->precision > IDF_PREC_I8) return fail(IDF_EINVAL, "unknown precision %d", d->precision);
    if (d->in_d < 1 || d->in_h < 1 || d->in_w < 1 || d->in_c < 1)
        return fail(IDF_EINVAL, "bad input shape %d x %d x %d x %d", d->in_d, d->in_h, d->in_w, d->in_c);
    // The column axis goes into the channels: position (row) x channel (column, c).  A layer's weights
    // become [(w_o, c_out)][(w_i, c_in)][k_d][k_h] with the entry of (w_i, w_o) taken from tap
    // kw = w_i - (w_o * s_w - p_w) where that is a tap, zero elsewhere; the bias is repeated per column.
    std::vector<idf_layer> lt(d->n_layers);
    std::vector<std::vector<unsigned char>> wt(d->n_layers), bt(d->n_layers);
    std::vector<const void *> wp(d->n_layers, nullptr), bp(d->n_layers, nullptr);
    const size_t wb = (size_t)w_bytes(d->precision);
    int w_in = d->in_w, c = d->in_c;
    for (int l = 0; l < d->n_layers; ++l) {
        const idf_volume_layer &L = d->layers[l];
        if (L.c_in != c || L.c_out < 1) return fail(IDF_EINVAL, "layer %d: c_in %d does not follow %d channels", l, L.c_in, c);
        if (L.k_d < 1 || L.k_h < 1 || L.k_w < 1 || L.s_d < 1 || L.s_h < 1 || L.s_w < 1 || L.p_d < 0 || L.p_h < 0 || L.p_w < 0)
            return fail(IDF_EINVAL, "layer %d: bad kernel/stride/padding", l);
        if (!weights || !weights[l]) return fail(IDF_EINVAL, "layer %d: no weights", l);
        const int w_out = out_size(w_in, L.k_w, L.s_w, L.p_w);
        if (w_out < 1) return fail(IDF_EINVAL, "layer %d: window larger than its input", l);
        const int64_t ci_f = (int64_t)w_in * L.c_in, co_f = (int64_t)w_out * L.c_out;
        if (ci_f > 4096 || co_f > 4096 || ci_f * co_f * L.k_d * L.k_h > ((int64_t)1 << 26))
            return fail(IDF_EUNSUPPORTED, "layer %d: %lld x %lld folded channels", l, (long long)ci_f, (long long)co_f);
        idf_layer &T = lt[l];
        T = idf_layer{};
        T.kind = IDF_CONV; T.c_in = (int)ci_f; T.c_out = (int)co_f;
        T.k_h = L.k_d; T.k_w = L.k_h; T.s_h = L.s_d; T.s_w = L.s_h; T.p_h = L.p_d; T.p_w = L.p_h;
        T.act = L.act; T.shr = L.shr; T.clamp_hi = L.clamp_hi;
        try { wt[l].assign((size_t)co_f * ci_f * L.k_d * L.k_h * wb, 0); }
        catch (const std::bad_alloc &) { return fail(IDF_ENOMEM, "out of host memory"); }
        const unsigned char *src = (const unsigned char *)weights[l];
        for (int wo = 0; wo < w_out; ++wo)
            for (int kw = 0; kw < L.k_w; ++kw) {
                const int wi = wo * L.s_w - L.p_w + kw;
                if (wi < 0 || wi >= w_in) continue;
                for (int co = 0; co < L.c_out; ++co)
                    for (int ci = 0; ci < L.c_in; ++ci)
                        for (int kd = 0; kd < L.k_d; ++kd)
                            for (int kh = 0; kh < L.k_h; ++kh) {
                                const size_t s_idx = ((((size_t)co * L.c_in + ci) * L.k_d + kd) * L.k_h + kh) * L.k_w + kw;
                                const size_t d_idx = ((((size_t)wo * L.c_out + co) * ci_f + (size_t)wi * L.c_in + ci) * L.k_d + kd) * L.k_h + kh;
                                memcpy(&wt[l][d_idx * wb], src + s_idx * wb, wb);
                            }
            }
        wp[l] = wt[l].data();
        if (biases && biases[l]) {
            bt[l].resize((size_t)co_f * 4);
            for (int wo = 0; wo < w_out; ++wo) memcpy(&bt[l][(size_t)wo * L.c_out * 4], biases[l], (size_t)L.c_out * 4);
            bp[l] = bt[l].data();
        }
        w_in = w_out; c = L.c_out;
    }
    idf_net_desc t{};
    t.precision = d->precision; t.in_h = d->in_d; t.in_w = d->in_h; t.in_c = d->in_w * d->in_c;
    t.n_layers = d->n_layers; t.layers = lt.data();
    return idf_create_net(&t, wp.data(), biases ? bp.data() : nullptr, out);
}

int idf_destroy_net(idf_net *net)
{
    if (!net) return IDF_OK;
    if (net->open_count > 0) return fail(IDF_ESTATE, "net still has %d open stream sets", net->open_count);
    delete net;
    return IDF_OK;
}

int idf_query_sizes(const idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows, idf_sizes *out)
{
    if (!net || !out) return fail(IDF_EINVAL, "null argument");
    if (n_streams < 1 || max_seg_rows < 1) return fail(IDF_EINVAL, "n_streams and max_seg_rows must be >= 1");
    Layout L;
    int rc = make_layout(*net, n_streams, max_seg_rows, out_cap_rows, L);
    if (rc != IDF_OK) return rc;
    *out = L.sizes;
    return IDF_OK;
}

int idf_open_streams(idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows, void *dev_workspace,
                     size_t workspace_bytes, void *hip_stream, idf_streams **out)
{
    if (!net || !out || !dev_workspace) return fail(IDF_EINVAL, "null argument");
    *out = nullptr;
    if (n_streams < 1 || max_seg_rows < 1) return fail(IDF_EINVAL, "n_streams and max_seg_rows must be >= 1");
    if (((uintptr_t)dev_workspace & 255) != 0) return fail(IDF_EINVAL, "workspace must be 256-byte aligned");
    Layout L;
    int rc = make_layout(*net, n_streams, max_seg_rows, out_cap_rows, L);
    if (rc != IDF_OK) return rc;
    if (workspace_bytes < L.total) return fail(IDF_EINVAL, "workspace of %zu bytes, %zu needed", workspace_bytes, L.total);
    return open_on(net, n_streams, max_seg_rows, out_cap_rows, L, dev_workspace, workspace_bytes, hip_stream, out);
}

int idf_open_streams_static(idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows, void *hip_stream,
                            idf_streams **out)
{
    if (!net || !out) return fail(IDF_EINVAL, "null argument");
    *out = nullptr;
    if (n_streams < 1 || max_seg_rows < 1) return fail(IDF_EINVAL, "n_streams and max_seg_rows must be >= 1");
    Layout L;
    int rc = make_layout(*net, n_streams, max_seg_rows, out_cap_rows, L);
    if (rc != IDF_OK) return rc;
    if (L.total > kStaticScratchBytes)
        return fail(IDF_ENOMEM, "these streams need a workspace of %zu bytes, the static one holds %zu: fewer streams, "
                                "or idf_open_streams with a workspace of the caller's", L.total, kStaticScratchBytes);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return dev_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(IDF_EDEVICE, "device %d outside the %d this library keeps a static workspace for", dev, kMaxDevices);
    unsigned char *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        StaticScratch &sc = g_scratch[dev];
        if (!sc.ptr) {
            // this device's copy of the array: its address, asked for with the device current
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return dev_fail(e, "hipGetSymbolAddress(scratch)");
            sc.ptr = (unsigned char *)p;
        }
        if (sc.in_use) return fail(IDF_ESTATE, "the static workspace of device %d is taken by another set of open streams", dev);
        sc.in_use = true;
        ws = sc.ptr;
    }
    // open_on clears every byte it lays out (the array keeps what the previous streams left there)
    rc = open_on(net, n_streams, max_seg_rows, out_cap_rows, L, ws, kStaticScratchBytes, hip_stream, out);
    if (rc != IDF_OK) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        g_scratch[dev].in_use = false;
        return rc;
    }
    (*out)->static_dev = dev;
    return IDF_OK;
}

int idf_close_streams(idf_streams *s)
{
    if (!s) return IDF_OK;
    (void)pipeline_drain(s);
    hipError_t e = hipStreamSynchronize(s->st);
    for (ProfRec &r : s->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (hipEvent_t ev : s->ev_pool) (void)hipEventDestroy(ev);
    if (s->static_dev >= 0) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        g_scratch[s->static_dev].in_use = false;
    }
    s->net->open_count--;
    delete s;
    return e == hipSuccess ? IDF_OK : dev_fail(e, "close_streams");
}

}  // extern "C"

namespace {

// Binds n_streams streams to a workspace laid out by L: host bookkeeping, upload of the packed
// weights, every laid-out byte cleared.
int open_on(idf_net *net, int n_streams, int max_seg_rows, int64_t out_cap_rows, const Layout &L, void *dev_workspace,
            size_t workspace_bytes, void *hip_stream, idf_streams **out)
{
    idf_streams *s = new (std::nothrow) idf_streams;
    if (!s) return fail(IDF_ENOMEM, "out of host memory");
    s->net = net; s->B = n_streams; s->max_seg = max_seg_rows;
    s->out_cap = out_cap_rows > 0 ? out_cap_rows : net->out_h;
    s->st = (hipStream_t)hip_stream; s->ws = (char *)dev_workspace; s->ws_bytes = workspace_bytes;
    s->w_off = L.w_off; s->b_off = L.b_off; s->wm_off = L.wm_off; s->ring_off = L.ring_off; s->held_off = L.held_off;
    s->transit_off = L.transit_off; s->ring_stride = L.ring_stride; s->held_stride = L.held_stride;
    s->transit_stride = L.transit_stride; s->transit_cap = L.transit_cap;
    s->out_off = L.out_off; s->stats_off = L.stats_off; s->issued_off = L.issued_off; s->out_stride = L.out_stride; s->sizes = L.sizes;
    s->use_cascade1d = L.cascade1d;
    s->head_off = L.head_off;
    s->cas_transit_off = L.cas_transit_off;
    s->cas_transit_stride = L.cas_transit_stride;
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&s->cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) s->cus = 0;
    }
    if (L.cascade1d) { plan_cascade_stages(s); cascade_layers(s); }
    s->mfma.assign(net->g.size(), 0);
    if (!getenv("IDF_NO_MFMA")) {
        for (size_t l = 0; l < net->g.size(); ++l) {
            if (net->wm_img[l].empty()) continue;
            s->mfma[l] = 1;
            if (l + 1 < net->g.size() && net->g[l + 1].kind == IDF_MAXPOOL && net->g[l + 1].k_w == 2) s->mfma[l + 1] = 2;
        }
    }
    s->stg2d = !strict_rows() && net_all_mfma(*net);
    if (s->stg2d) {
        for (size_t l = 0; l < net->g.size(); ++l)
            if (net->g[l].kind == IDF_CONV) s->stg_unit.push_back((int)l);
        s->stg_fifo.assign(s->stg_unit.size(), {});
        // One tile shape for all layers of a launch: 32 positions (measured faster than 64 on every
        // workload: rows of 224 or 112 positions waste less, and the smaller workgroups of a
        // launch overlap better), 32 channels when some layer has no more.
        int c_min = 1 << 30;
        for (int l : s->stg_unit) c_min = std::min(c_min, net->g[l].c_out);
        s->stg_tile = c_min > 32 ? kMfmaTile32x64 : kMfmaTile32x32;
        s->stg_seq.assign(s->stg_unit.size(), 0);
        s->stg_slots = max_seg_rows >= 2 ? 2 * kStgSlots : kStgSlots;
        s->stg_pairs = max_seg_rows >= 2 && !getenv("IDF_NO_ROW_PAIRS");
    }
    s->h.assign(n_streams, StreamHost{});
    s->stamp.assign(n_streams, 0);
    hipError_t e = launch_fill_zero(s->ws, L.sizes.weights_bytes, s->st);     // zero padding of the weights
    for (size_t l = 0; l < net->g.size() && e == hipSuccess; ++l) {
        if (net->g[l].kind != IDF_CONV) continue;
        if (L.cascade1d) {
            const Geom &g = net->g[l];
            const float *src = (const float *)net->w_img[l].data();      // [k_h][1][c_in][c_out]
            s->cas_w.emplace_back((size_t)cascade1d_cin_pad(g.c_in, g.c_out) * g.c_out * kCasKMax, 0.f);
            std::vector<float> &img = s->cas_w.back();
            for (int ky = 0; ky < g.k_h; ++ky)
                for (int ci = 0; ci < g.c_in; ++ci)
                    for (int co = 0; co < g.c_out; ++co)
                        img[cascade1d_weight_index(g.c_in, g.c_out, ci, co, ky)] = src[((size_t)ky * g.c_in + ci) * g.c_out + co];
            e = hipMemcpyAsync(s->ws + s->w_off[l], img.data(), img.size() * 4, hipMemcpyHostToDevice, s->st);
        } else {
            e = hipMemcpyAsync(s->ws + s->w_off[l], net->w_img[l].data(), net->w_img[l].size(), hipMemcpyHostToDevice, s->st);
        }
        if (e == hipSuccess && !net->b_img[l].empty())
            e = hipMemcpyAsync(s->ws + s->b_off[l], net->b_img[l].data(), net->b_img[l].size(), hipMemcpyHostToDevice, s->st);
        if (e == hipSuccess && !net->wm_img[l].empty())
            e = hipMemcpyAsync(s->ws + s->wm_off[l], net->wm_img[l].data(), net->wm_img[l].size(), hipMemcpyHostToDevice, s->st);
    }
    // State needs no clearing for correctness (a row of c is initialised when first touched);
    // it is zeroed once so that the workspace never exposes stale bytes.
    if (e == hipSuccess)
        e = launch_fill_zero(s->ws + L.sizes.weights_bytes, L.total - L.sizes.weights_bytes, s->st);
    if (e != hipSuccess) { delete s; return dev_fail(e, "open_streams"); }
    net->open_count++;
    *out = s;
    return IDF_OK;
}

}  // namespace

extern "C" {

int idf_push_segment(idf_streams *s, const int32_t *stream_ids, int n_ids, const void *dev_rows, int n_rows)
{
    if (!s || !dev_rows) return fail(IDF_EINVAL, "null argument");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    if (n_rows < 1 || n_rows > s->max_seg) return fail(IDF_EINVAL, "n_rows %d outside [1, %d]", n_rows, s->max_seg);
    if (s->eager.on) return eager_push(s, stream_ids, n_ids, dev_rows, n_rows);
    const idf_net &net = *s->net;
    // Validate everything before anything is enqueued.  Streams pushed in step -- the usual case --
    // share one row number and one output slot: they form one group, found without building the
    // map, and what depends on the row number only is worked out once per distinct value.
    std::vector<std::pair<int, int>> &members = s->push_members;
    members.clear();
    std::pair<int64_t, int64_t> key0{0, 0};
    bool one_group = true;
    int64_t memo_r = -1, memo_fresh = 0;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        const StreamHost &h = s->h[id];
        if (h.x_next != 0 && !s->part.on)
            return fail(IDF_ESTATE, "stream %d: %d columns of a row were pushed as pixels, the row must be finished that way", id, h.x_next);
        if (net.in_h > 0 && h.r + n_rows > net.in_h)
            return fail(IDF_ESTATE, "stream %d: rows %lld..%lld run past the sample of %d rows", id,
                        (long long)h.r, (long long)(h.r + n_rows - 1), net.in_h);
        if (h.r != memo_r) { memo_r = h.r; memo_fresh = output_rows_of_push(net, h.r, n_rows); }
        const int64_t fresh = memo_fresh;
        if (h.out_written - h.out_read + fresh > s->out_cap)
            return fail(IDF_ESTATE, "stream %d: output area full (%lld rows waiting, %lld more would complete, room for %lld)",
                        id, (long long)(h.out_written - h.out_read), (long long)fresh, (long long)s->out_cap);
        const std::pair<int64_t, int64_t> key{h.r, h.out_written % s->out_cap};
        if (i == 0) key0 = key;
        else if (key != key0) one_group = false;
        members.push_back({i, id});
    }
    if (one_group) {
        rc = for_each_selection(members, [&](const StreamSel &sel) {
            return enqueue_cascade(s, sel, dev_rows, n_rows, key0.first, key0.second);
        });
        if (rc != IDF_OK) return rc;
    } else {
        std::map<std::pair<int64_t, int64_t>, std::vector<std::pair<int, int>>> groups;
        for (const auto &m : members) {
            const StreamHost &h = s->h[m.second];
            groups[{h.r, h.out_written % s->out_cap}].push_back(m);
        }
        for (auto &kv : groups) {
            const int64_t r = kv.first.first, slot0 = kv.first.second;
            rc = for_each_selection(kv.second, [&](const StreamSel &sel) {
                return enqueue_cascade(s, sel, dev_rows, n_rows, r, slot0);
            });
            if (rc != IDF_OK) return rc;
        }
    }
    memo_r = -1;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        StreamHost &h = s->h[id];
        if (h.r != memo_r) { memo_r = h.r; memo_fresh = output_rows_of_push(net, h.r, n_rows); }
        h.out_written += memo_fresh;
        h.r += n_rows;
        h.x_next = 0;
        if (net.in_h > 0 && h.r == net.in_h) h.r = 0;      // next sample
    }
    return IDF_OK;
}

int idf_push_pixels(idf_streams *s, const int32_t *stream_ids, int n_ids, const void *dev_pixels, int x0, int n_px)
{
    if (!s || !dev_pixels) return fail(IDF_EINVAL, "null argument");
    const idf_net &net = *s->net;
    if (n_px < 1 || x0 < 0 || x0 + n_px > net.in_w) return fail(IDF_EINVAL, "columns %d..%d outside the row of %d", x0, x0 + n_px - 1, net.in_w);
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "pixel segments are not built for eager emission");
    if (x0 == 0 && n_px == net.in_w) return idf_push_segment(s, stream_ids, n_ids, dev_pixels, 1);
    const bool first_mfma = !s->mfma.empty() && s->mfma[0] == 1;
    if (net.g[0].kind != IDF_CONV) return fail(IDF_EUNSUPPORTED, "pixel segments need a convolution as the first layer");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        if (s->h[id].x_next != x0)
            return fail(IDF_ESTATE, "stream %d: next column is %d, not %d", id, s->h[id].x_next, x0);
    }
    s->part.on = true; s->part.x_lo = x0; s->part.x_hi = x0 + n_px; s->part.first = x0 == 0; s->part.last = x0 + n_px == net.in_w;
    if (s->part.last) {
        // the row is whole: everything a pushed row does, with layer 0 taking only these columns
        rc = idf_push_segment(s, stream_ids, n_ids, dev_pixels, 1);
        s->part = idf_streams::Part{};
        return rc;
    }
    // layer 0 takes the columns into its rolling buffer; nothing can be final yet
    std::map<int64_t, std::vector<std::pair<int, int>>> groups;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        if (net.in_h > 0 && s->h[id].r >= net.in_h) { s->part = idf_streams::Part{}; return fail(IDF_ESTATE, "stream %d: sample complete", id); }
        groups[s->h[id].r].push_back({i, id});
    }
    for (auto &kv : groups) {
        const int64_t r = kv.first;
        rc = for_each_selection(kv.second, [&](const StreamSel &sel) {
            if (!first_mfma) {
                // any other first convolution: the generic kernel with the segment's column range; every row the input
                // row touches goes back to the rolling buffer
                const Geom &g = net.g[0];
                ConvStep c{};
                c.g = g; c.layer = 0; c.y0 = r; c.cnt = 1;
                c.o_lo = rows_final(g, r); c.o_fin = c.o_lo;
                c.o_hi = std::max(rows_touched(g, r + 1), rows_final(g, r + 1));
                if (c.o_hi <= c.o_lo) return (int)IDF_OK;          // the row reaches no output row (stride and padding skip it)
                c.ring_rows = g.k_h;
                c.in = dev_pixels; c.in_stream_stride = (int64_t)n_px * net.in_c; c.in_row0 = r; c.in_by_position = 1;
                c.ring = s->ws + s->ring_off[0]; c.ring_stream_stride = s->ring_stride[0];
                c.dst = nullptr; c.dst_row0 = c.o_lo; c.out_cap = s->out_cap;
                c.w = s->ws + s->w_off[0];
                c.bias = net.b_img[0].empty() ? nullptr : s->ws + s->b_off[0];
                c.stats = (unsigned long long *)(s->ws + s->stats_off); c.n_layers = (int)net.g.size();
                c.x_lo = x0; c.x_hi = x0 + n_px; c.cont = x0 != 0;
                conv_generic_plan(c);
                hipError_t e = launch_conv_generic(net.precision, c, sel, launch_ctx(s, kKindConvGeneric, conv_step_bytes(net, c, sel.n), 0));
                return e == hipSuccess ? (int)IDF_OK : dev_fail(e, "pixel segment launch");
            }
            MfmaStep a;
            int64_t rows_out[3];
            double bytes = 0;
            make_mfma_step(s, 0, r, sel.n, a, rows_out, bytes);
            a.in = dev_pixels; a.in_stream_stride = (int64_t)n_px * net.in_c; a.in_by_position = 1;
            a.in_row_off = -(int64_t)x0 * net.in_c;
            hipError_t e = launch_conv3x3_mfma(net.precision, a, sel, launch_ctx(s, kKindConvMfma, bytes, 0));
            return e == hipSuccess ? IDF_OK : dev_fail(e, "pixel segment launch");
        });
        if (rc != IDF_OK) break;
    }
    s->part = idf_streams::Part{};
    if (rc != IDF_OK) return rc;
    for (int i = 0; i < n_ids; ++i) s->h[stream_ids ? stream_ids[i] : i].x_next = x0 + n_px;
    return IDF_OK;
}

int idf_read_outputs(idf_streams *s, const int32_t *stream_ids, int n_ids, void *dev_out, int64_t max_rows,
                     int64_t *first_row, int32_t *n_rows)
{
    if (!s || !dev_out || !first_row || !n_rows) return fail(IDF_EINVAL, "null argument");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    if (max_rows < 1) return fail(IDF_EINVAL, "max_rows must be >= 1");
    if (s->eager.on) return fail(IDF_ESTATE, "eager emission: the output is read with idf_read_announced");
    rc = pipeline_drain(s);                // rows still between stages belong to what was pushed
    if (rc != IDF_OK) return rc;
    rc = head_catch_up(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    const idf_net &net = *s->net;
    std::map<std::pair<int64_t, int>, std::vector<std::pair<int, int>>> groups;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        const StreamHost &h = s->h[id];
        const int64_t n = std::min<int64_t>(h.out_written - h.out_read, max_rows);
        first_row[i] = net.out_h > 0 ? h.out_read % net.out_h : h.out_read;
        n_rows[i] = (int32_t)n;
        if (n > 0) groups[{h.out_read % s->out_cap, (int)n}].push_back({i, id});
    }
    CopyOut a{};
    a.src = s->ws + s->out_off; a.src_stream_stride = s->out_stride; a.out_cap = s->out_cap;
    a.dst = dev_out; a.row_elems = (int64_t)net.out_w * net.out_c; a.dst_stream_stride = max_rows * a.row_elems;
    a.elem_bytes = 4;
    for (auto &kv : groups) {
        const int64_t slot = kv.first.first;
        const int n = kv.first.second;
        rc = for_each_selection(kv.second, [&](const StreamSel &sel) {
            hipError_t e = launch_copy_out(a, sel, slot, n,
                                           launch_ctx(s, kKindCopyOut, 8.0 * n * a.row_elems * sel.n));
            return e == hipSuccess ? IDF_OK : dev_fail(e, "copy launch");
        });
        if (rc != IDF_OK) return rc;
    }
    for (int i = 0; i < n_ids; ++i) s->h[stream_ids ? stream_ids[i] : i].out_read += n_rows[i];
    return IDF_OK;
}

int idf_reset_streams(idf_streams *s, const int32_t *stream_ids, int n_ids)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    rc = pipeline_drain(s);
    if (rc != IDF_OK) return rc;
    const size_t per = s->net->g.size() * 2 * sizeof(unsigned long long);
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        hipError_t e = launch_fill_zero(s->ws + s->stats_off + per * id, per, s->st);
        if (e == hipSuccess) e = launch_fill_zero(s->ws + s->issued_off + per / 2 * id, per / 2, s->st);
        if (e == hipSuccess)
            e = launch_fill_zero(s->ws + s->head_off + (size_t)id * s->net->out_c * sizeof(double),
                                 (size_t)s->net->out_c * sizeof(double), s->st);
        if (e != hipSuccess) return dev_fail(e, "reset_streams");
        s->h[id] = StreamHost{};
    }
    return IDF_OK;
}

int idf_get_stats(idf_streams *s, int stream_id, uint64_t *events_in, uint64_t *macs_executed, uint64_t *state_bytes)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    if (stream_id < 0 || stream_id >= s->B) return fail(IDF_EINVAL, "stream id %d outside [0, %d)", stream_id, s->B);
    const int n = (int)s->net->g.size();
    std::vector<unsigned long long> buf((size_t)n * 2);
    if (int rc = pipeline_drain(s)) return rc;
    hipError_t e = hipStreamSynchronize(s->st);
    if (e == hipSuccess)
        e = hipMemcpy(buf.data(), s->ws + s->stats_off + (size_t)stream_id * n * 2 * sizeof(unsigned long long),
                      buf.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return dev_fail(e, "get_stats");
    const int eb = ev_bytes(s->net->precision);
    for (int l = 0; l < n; ++l) {
        if (events_in) events_in[l] = buf[2 * l];
        if (macs_executed) macs_executed[l] = buf[2 * l + 1];
        if (state_bytes)
            state_bytes[l] = s->net->g[l].kind == IDF_CONV ? (uint64_t)s->ring_stride[l] * 4 : (uint64_t)s->held_stride[l] * eb;
    }
    return IDF_OK;
}

int idf_count_issued_macs(idf_streams *s, int on)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "eager emission keeps no count of issued multiply-adds");
    int rc = pipeline_drain(s);                 // what is on its way was pushed under the old setting
    if (rc != IDF_OK) return rc;
    s->count_issued = on != 0;
    return IDF_OK;
}

int idf_set_event_path(idf_streams *s, int events_per_kstep)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    if (events_per_kstep < 0) return fail(IDF_EINVAL, "events per K-step %d is negative", events_per_kstep);
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "eager emission has one kernel per layer kind and no event-list variant");
    int rc = pipeline_drain(s);                 // what is on its way was pushed under the old setting
    if (rc != IDF_OK) return rc;
    s->ev_per_step = std::min(events_per_kstep, 1 << 16);
    return IDF_OK;
}

int idf_get_issued_macs(idf_streams *s, int stream_id, uint64_t *macs_issued)
{
    if (!s || !macs_issued) return fail(IDF_EINVAL, "null argument");
    if (stream_id < 0 || stream_id >= s->B) return fail(IDF_EINVAL, "stream id %d outside [0, %d)", stream_id, s->B);
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "eager emission keeps no count of issued multiply-adds");
    const int n = (int)s->net->g.size();
    std::vector<unsigned long long> iss((size_t)n), st((size_t)n * 2);
    if (int rc = pipeline_drain(s)) return rc;
    hipError_t e = hipStreamSynchronize(s->st);
    if (e == hipSuccess)
        e = hipMemcpy(iss.data(), s->ws + s->issued_off + (size_t)stream_id * n * sizeof(unsigned long long),
                      iss.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
    if (e == hipSuccess)
        e = hipMemcpy(st.data(), s->ws + s->stats_off + (size_t)stream_id * n * 2 * sizeof(unsigned long long),
                      st.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return dev_fail(e, "get_issued_macs");
    // the generic kernels test every value and keep no count of their own: they issue what they execute
    const bool own_count = s->use_cascade1d || !s->mfma.empty();
    for (int l = 0; l < n; ++l) {
        const bool counted = s->use_cascade1d || (own_count && l < (int)s->mfma.size() && s->mfma[l] == 1);
        macs_issued[l] = counted ? iss[l] : st[2 * l + 1];
    }
    return IDF_OK;
}

int idf_set_push_batching(idf_streams *s, int k)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    if (k < 1 || k > kCasSegMax) return fail(IDF_EINVAL, "pushes per launch %d outside [1, %d]", k, kCasSegMax);
    if (!s->use_cascade1d) return fail(IDF_EUNSUPPORTED, "holding back pushes is built for nets served by the 1-D cascade");
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "eager emission delivers every segment at once");
    int rc = pipeline_drain(s);                  // what is held back was pushed under the old setting
    if (rc != IDF_OK) return rc;
    s->cas_batch = k;
    return IDF_OK;
}

int idf_rows_pushed(const idf_streams *s, int stream_id, int64_t *rows)
{
    if (!s || !rows) return fail(IDF_EINVAL, "null argument");
    if (stream_id < 0 || stream_id >= s->B) return fail(IDF_EINVAL, "stream id %d outside [0, %d)", stream_id, s->B);
    *rows = s->h[stream_id].r;
    return IDF_OK;
}

int idf_snapshot_bytes(const idf_streams *s, size_t *bytes)
{
    if (!s || !bytes) return fail(IDF_EINVAL, "null argument");
    size_t total = 0;
    for_each_state_piece(s, 0, [&](size_t, size_t n) { total += align_up(n, 16); });
    *bytes = total;
    return IDF_OK;
}

int idf_snapshot(idf_streams *s, int stream_id, void *dev_buf, idf_stream_pos *pos)
{
    if (!s || !dev_buf || !pos) return fail(IDF_EINVAL, "null argument");
    if (stream_id < 0 || stream_id >= s->B) return fail(IDF_EINVAL, "stream id %d outside [0, %d)", stream_id, s->B);
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "snapshots do not cover the maps of eager emission");
    if (s->head_units) return fail(IDF_EUNSUPPORTED, "snapshots do not cover the fully connected output units");
    if (s->h[stream_id].x_next != 0) return fail(IDF_ESTATE, "stream %d: a row is half presented", stream_id);
    int rc = pipeline_drain(s);
    if (rc != IDF_OK) return rc;
    const int32_t id32 = stream_id;
    rc = head_catch_up(s, &id32, 1);
    if (rc != IDF_OK) return rc;
    const StreamHost &h = s->h[stream_id];
    if (h.out_written != h.out_read) return fail(IDF_ESTATE, "stream %d: %lld completed output rows not read yet", stream_id,
                                                 (long long)(h.out_written - h.out_read));
    size_t at = 0;
    hipError_t e = hipSuccess;
    for_each_state_piece(s, stream_id, [&](size_t off, size_t n) {
        if (e == hipSuccess && n) e = hipMemcpyAsync((char *)dev_buf + at, s->ws + off, n, hipMemcpyDeviceToDevice, s->st);
        at += align_up(n, 16);
    });
    if (e != hipSuccess) return dev_fail(e, "snapshot");
    pos->rows_pushed = h.r; pos->out_rows = h.out_written; pos->head_rows = h.head_done - h.head_base;
    return IDF_OK;
}

int idf_restore(idf_streams *s, int stream_id, const void *dev_buf, const idf_stream_pos *pos)
{
    if (!s || !dev_buf || !pos) return fail(IDF_EINVAL, "null argument");
    if (stream_id < 0 || stream_id >= s->B) return fail(IDF_EINVAL, "stream id %d outside [0, %d)", stream_id, s->B);
    const idf_net &net = *s->net;
    if (pos->rows_pushed < 0 || (net.in_h > 0 && pos->rows_pushed >= net.in_h) || pos->out_rows < 0 ||
        pos->head_rows < 0 || pos->head_rows > pos->out_rows)
        return fail(IDF_EINVAL, "inconsistent stream position");
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "snapshots do not cover the maps of eager emission");
    if (s->head_units) return fail(IDF_EUNSUPPORTED, "snapshots do not cover the fully connected output units");
    int rc = pipeline_drain(s);
    if (rc != IDF_OK) return rc;
    StreamHost &h = s->h[stream_id];
    if (h.out_written != h.out_read) return fail(IDF_ESTATE, "stream %d: %lld completed output rows not read yet", stream_id,
                                                 (long long)(h.out_written - h.out_read));
    size_t at = 0;
    hipError_t e = hipSuccess;
    for_each_state_piece(s, stream_id, [&](size_t off, size_t n) {
        if (e == hipSuccess && n) e = hipMemcpyAsync(s->ws + off, (const char *)dev_buf + at, n, hipMemcpyDeviceToDevice, s->st);
        at += align_up(n, 16);
    });
    if (e != hipSuccess) return dev_fail(e, "restore");
    h.r = pos->rows_pushed; h.out_written = h.out_read = pos->out_rows; h.x_next = 0;
    h.head_done = pos->out_rows; h.head_base = pos->out_rows - pos->head_rows;
    return IDF_OK;
}

int idf_query_eager_bytes(const idf_net *net, int n_streams, int max_seg_rows, size_t *bytes)
{
    if (!net || !bytes || n_streams < 1 || max_seg_rows < 1) return fail(IDF_EINVAL, "bad argument");
    if (net->in_h <= 0) return fail(IDF_EUNSUPPORTED, "eager emission keeps the output map whole: the sample height must be known");
    *bytes = eager_layout(*net, n_streams, max_seg_rows, nullptr);
    return IDF_OK;
}

int idf_enable_eager(idf_streams *s, void *dev_workspace, size_t workspace_bytes)
{
    if (!s || !dev_workspace) return fail(IDF_EINVAL, "null argument");
    size_t need = 0;
    int rc = idf_query_eager_bytes(s->net, s->B, s->max_seg, &need);
    if (rc != IDF_OK) return rc;
    if (workspace_bytes < need) return fail(IDF_EINVAL, "eager workspace of %zu bytes, %zu needed", workspace_bytes, need);
    if (s->head_on) return fail(IDF_EUNSUPPORTED, "the averaging units read completed rows, eager emission has none");
    for (const StreamHost &h : s->h)
        if (h.r != 0 || h.out_written != 0 || h.x_next != 0) return fail(IDF_ESTATE, "eager emission must be enabled before the first push");
    eager_layout(*s->net, s->B, s->max_seg, &s->eager);
    s->eager.ws = (char *)dev_workspace;
    s->eager.on = true;
    return IDF_OK;
}

int idf_eager_state_bytes(const idf_streams *s, size_t *per_stream, int *rows_kept)
{
    if (!s || !per_stream) return fail(IDF_EINVAL, "null argument");
    if (!s->eager.on) return fail(IDF_ESTATE, "eager emission is not enabled");
    const idf_streams::Eager &E = s->eager;
    const int n = (int)s->net->g.size();
    size_t total = 0;
    for (int lv = 0; lv <= n; ++lv) {
        const bool has_c = lv > 0 && s->net->g[lv - 1].kind == IDF_CONV;
        // state c and the announced values; the deltas live only during a push, the last level's announced map is the output
        total += (size_t)E.row_elems[lv] * 4 * ((has_c ? E.cd_rows[lv] : 0) + (lv < n ? E.ann_rows[lv] : 0));
        if (rows_kept) rows_kept[lv] = E.cd_rows[lv];
    }
    *per_stream = total;
    return IDF_OK;
}

int idf_read_announced(idf_streams *s, int level, const int32_t *stream_ids, int n_ids, void *dev_out)
{
    if (!s || !dev_out) return fail(IDF_EINVAL, "null argument");
    if (!s->eager.on) return fail(IDF_ESTATE, "eager emission is not enabled");
    const int n = (int)s->net->g.size();
    if (level < 0 || level > n) return fail(IDF_EINVAL, "level %d outside [0, %d]", level, n);
    if (s->eager.ring && level != n)
        return fail(IDF_ESTATE, "level %d keeps a ring of %d rows, not its whole map: read them with idf_read_announced_rows", level,
                    s->eager.ann_rows[level]);
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    const size_t bytes = (size_t)s->eager.rows[level] * s->eager.row_elems[level] * 4;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        hipError_t e = hipMemcpyAsync((char *)dev_out + (size_t)i * bytes, s->eager.ws + s->eager.ann_off[level] + (size_t)id * bytes,
                                      bytes, hipMemcpyDeviceToDevice, s->st);
        if (e != hipSuccess) return dev_fail(e, "read_announced");
    }
    return IDF_OK;
}

int idf_read_announced_rows(idf_streams *s, int level, const int32_t *stream_ids, int n_ids, void *dev_out, int max_rows,
                            int64_t *first_row, int32_t *n_rows)
{
    if (!s || !dev_out || !first_row || !n_rows) return fail(IDF_EINVAL, "null argument");
    if (!s->eager.on) return fail(IDF_ESTATE, "eager emission is not enabled");
    const idf_streams::Eager &E = s->eager;
    const int n = (int)s->net->g.size();
    if (level < 0 || level > n) return fail(IDF_EINVAL, "level %d outside [0, %d]", level, n);
    if (max_rows < 1) return fail(IDF_EINVAL, "max_rows must be >= 1");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    const size_t row_bytes = (size_t)E.row_elems[level] * 4;
    std::vector<int64_t> lo, hi;
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        // rows of the level reached by the input rows seen so far; the newest `rows kept` of them are still there
        eager_bands(*s->net, 0, s->h[id].eager_rows, false, lo, hi);
        const bool whole = !E.ring || level == n;             // kept whole and cleared when the sample began
        const int64_t reached = whole ? (s->h[id].eager_rows > 0 ? E.rows[level] : 0) : hi[level];
        const int64_t first = whole ? 0 : std::max<int64_t>(0, reached - E.ann_rows[level]);
        const int64_t cnt = std::min<int64_t>(reached - first, max_rows);
        first_row[i] = first; n_rows[i] = (int32_t)cnt;
        const char *src = s->eager.ws + E.ann_off[level] + (size_t)id * E.ann_rows[level] * row_bytes;
        for (int64_t r = first; r < first + cnt; ++r) {         // (a ring wraps: row by row)
            hipError_t e = hipMemcpyAsync((char *)dev_out + ((size_t)i * max_rows + (size_t)(r - first)) * row_bytes,
                                          src + (size_t)(r % E.ann_rows[level]) * row_bytes, row_bytes, hipMemcpyDeviceToDevice, s->st);
            if (e != hipSuccess) return dev_fail(e, "read_announced_rows");
        }
    }
    return IDF_OK;
}

int idf_enable_head(idf_streams *s)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    if (s->eager.on) return fail(IDF_EUNSUPPORTED, "the averaging units read completed rows, eager emission has none");
    for (const StreamHost &h : s->h)
        if (h.r != 0 || h.out_written != 0) return fail(IDF_ESTATE, "the averaging units must be enabled before the first push");
    s->head_on = true;
    return IDF_OK;
}

int idf_query_head_units_bytes(const idf_net *net, int n_streams, int n_units, size_t *bytes)
{
    if (!net || !bytes || n_streams < 1 || n_units < 1) return fail(IDF_EINVAL, "bad argument");
    if (net->out_h <= 0) return fail(IDF_EUNSUPPORTED, "output units have one weight per position: the sample height must be known");
    const size_t map = (size_t)net->out_h * net->out_w * net->out_c;
    *bytes = align_up(((size_t)n_units * map + n_units) * 4) + align_up((size_t)n_streams * n_units * sizeof(double));
    return IDF_OK;
}

int idf_enable_head_units(idf_streams *s, int n_units, const float *weights, const float *bias, void *dev_buf, size_t bytes)
{
    if (!s || !weights || !dev_buf) return fail(IDF_EINVAL, "null argument");
    size_t need = 0;
    int rc = idf_query_head_units_bytes(s->net, s->B, n_units, &need);
    if (rc != IDF_OK) return rc;
    if (bytes < need) return fail(IDF_EINVAL, "buffer of %zu bytes for the output units, %zu needed", bytes, need);
    rc = idf_enable_head(s);                       // the units ride on the averaging units' bookkeeping
    if (rc != IDF_OK) return rc;
    const size_t map = (size_t)s->net->out_h * s->net->out_w * s->net->out_c;
    hipError_t e = launch_fill_zero(dev_buf, need, s->st);
    if (e == hipSuccess) e = hipMemcpyAsync(dev_buf, weights, (size_t)n_units * map * 4, hipMemcpyHostToDevice, s->st);
    if (e == hipSuccess && bias)
        e = hipMemcpyAsync((char *)dev_buf + (size_t)n_units * map * 4, bias, (size_t)n_units * 4, hipMemcpyHostToDevice, s->st);
    if (e == hipSuccess) e = hipStreamSynchronize(s->st);          // the host arrays may go after the call
    if (e != hipSuccess) return dev_fail(e, "enable_head_units");
    s->head_units = n_units; s->head_units_ws = (char *)dev_buf; s->head_units_bias = bias != nullptr;
    return IDF_OK;
}

int idf_read_head_units(idf_streams *s, const int32_t *stream_ids, int n_ids, double *values, int64_t *rows)
{
    if (!s || !values || !rows) return fail(IDF_EINVAL, "null argument");
    if (!s->head_units) return fail(IDF_ESTATE, "no output units enabled");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    rc = pipeline_drain(s);
    if (rc != IDF_OK) return rc;
    rc = head_catch_up(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    const int k = s->head_units;
    const size_t map = (size_t)s->net->out_h * s->net->out_w * s->net->out_c;
    std::vector<double> all((size_t)s->B * k);
    std::vector<float> b(k, 0.f);
    hipError_t e = hipStreamSynchronize(s->st);
    if (e == hipSuccess)
        e = hipMemcpy(all.data(), s->head_units_ws + align_up(((size_t)k * map + k) * 4), all.size() * sizeof(double), hipMemcpyDeviceToHost);
    if (e == hipSuccess && s->head_units_bias)
        e = hipMemcpy(b.data(), s->head_units_ws + (size_t)k * map * 4, (size_t)k * 4, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return dev_fail(e, "read_head_units");
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        rows[i] = s->h[id].head_done - s->h[id].head_base;
        // a unit that has received no row yet still states its bias (a constant input, Sec. 3)
        for (int u = 0; u < k; ++u) values[(size_t)i * k + u] = rows[i] > 0 ? all[(size_t)id * k + u] : (double)b[u];
    }
    return IDF_OK;
}

int idf_read_head(idf_streams *s, const int32_t *stream_ids, int n_ids, double *mean, int64_t *rows)
{
    if (!s || !mean || !rows) return fail(IDF_EINVAL, "null argument");
    if (!s->head_on) return fail(IDF_ESTATE, "the averaging units are not enabled");
    int rc = check_ids(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    rc = pipeline_drain(s);
    if (rc != IDF_OK) return rc;
    rc = head_catch_up(s, stream_ids, n_ids);
    if (rc != IDF_OK) return rc;
    const int c = s->net->out_c;
    std::vector<double> all((size_t)s->B * c);
    hipError_t e = hipStreamSynchronize(s->st);
    if (e == hipSuccess)
        e = hipMemcpy(all.data(), s->ws + s->head_off + (size_t)s->B * c * sizeof(double), all.size() * sizeof(double),
                      hipMemcpyDeviceToHost);
    if (e != hipSuccess) return dev_fail(e, "read_head");
    for (int i = 0; i < n_ids; ++i) {
        const int id = stream_ids ? stream_ids[i] : i;
        rows[i] = s->h[id].head_done - s->h[id].head_base;
        for (int k = 0; k < c; ++k) mean[(size_t)i * c + k] = rows[i] > 0 ? all[(size_t)id * c + k] : 0.0;
    }
    return IDF_OK;
}

int idf_measure_peak(int kind, void *dev_buf, size_t bytes, void *hip_stream, double *rate)
{
    if (!dev_buf || !rate) return fail(IDF_EINVAL, "null argument");
    if (kind < IDF_PEAK_COPY || kind > IDF_PEAK_MFMA_I8) return fail(IDF_EINVAL, "unknown kind %d", kind);
    int dev = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess || cus < 1) return dev_fail(e, "measure_peak: device query");
    const bool copy = kind == IDF_PEAK_COPY;
    const int blocks = copy ? cus * 8 : cus * 2;             // two workgroups of four waves per compute unit: two waves per SIMD
    const int iters = 2048;
    if (bytes < ((size_t)1 << 20) || bytes < peak_sink_bytes(blocks))
        return fail(IDF_EINVAL, "measure_peak: the buffer holds %zu bytes, at least %zu are needed", bytes,
                    std::max<size_t>((size_t)1 << 20, peak_sink_bytes(blocks)));
    hipStream_t st = (hipStream_t)hip_stream;
    LaunchCtx lc;
    lc.st = st;
    e = launch_peak(kind, dev_buf, bytes, blocks, iters, lc);     // untimed: code and clocks warm
    hipEvent_t a = nullptr, b = nullptr;
    if (e == hipSuccess) e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    float best = 0.f;
    for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
        lc.start = a; lc.stop = b;
        e = launch_peak(kind, dev_buf, bytes, blocks, iters, lc);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e == hipSuccess && (best == 0.f || ms < best)) best = ms;
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (e != hipSuccess) return dev_fail(e, "measure_peak");
    if (best <= 0.f) return fail(IDF_EDEVICE, "measure_peak: no time was measured");
    const double work = copy ? 2.0 * (double)(bytes / 32 * 16) : peak_ops(kind, blocks, iters);
    *rate = work / ((double)best * 1e-3) / (copy ? 1e9 : 1e12);
    return IDF_OK;
}

int idf_profile_begin(idf_streams *s)
{
    if (!s) return fail(IDF_EINVAL, "null argument");
    if (s->prof_on) return fail(IDF_ESTATE, "profiling already on");
    s->prof_on = true;
    return IDF_OK;
}

int idf_profile_end(idf_streams *s, int max_kinds, idf_kernel_profile *out, int *n_kinds)
{
    if (!s || !out || !n_kinds || max_kinds < 1) return fail(IDF_EINVAL, "null argument");
    if (!s->prof_on) return fail(IDF_ESTATE, "profiling is not on");
    if (int rc = pipeline_drain(s)) return rc;
    s->prof_on = false;
    hipError_t e = hipStreamSynchronize(s->st);
    if (e != hipSuccess) return dev_fail(e, "profile_end");
    struct Agg { double ms = 0, bytes = 0; uint64_t cnt = 0; };
    std::map<std::pair<int, int>, Agg> agg;
    for (ProfRec &r : s->prof) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) {
            Agg &g = agg[{r.kind, r.layer}];
            g.ms += t; g.bytes += r.bytes; g.cnt++;
        }
        s->ev_pool.push_back(r.a); s->ev_pool.push_back(r.b);
    }
    s->prof.clear();
    int n = 0;
    for (auto &kv : agg) {
        if (n >= max_kinds) break;
        memset(&out[n], 0, sizeof(out[n]));
        if (kv.first.second >= 0) snprintf(out[n].name, sizeof(out[n].name), "%s@%d", kind_name(kv.first.first), kv.first.second);
        else snprintf(out[n].name, sizeof(out[n].name), "%s", kind_name(kv.first.first));
        out[n].launches = kv.second.cnt; out[n].total_ms = kv.second.ms; out[n].algorithmic_bytes = kv.second.bytes;
        ++n;
    }
    *n_kinds = n;
    return IDF_OK;
}

const char *idf_layer_kernel(const idf_streams *s, int layer)
{
    if (!s || layer < 0 || layer >= (int)s->net->g.size()) return nullptr;
    if (s->use_cascade1d) return kind_name(kKindCascade1d);
    if (s->mfma[layer]) return kind_name(kKindConvMfma);
    return s->net->g[layer].kind == IDF_CONV ? kind_name(kKindConvGeneric) : kind_name(kKindPoolGeneric);
}

}  // extern "C"
