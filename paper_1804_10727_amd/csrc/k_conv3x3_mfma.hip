// Matrix-core event propagation for one arriving row of a 3x3, stride 1, same-padded conv layer
// (bfloat16 events and weights -> float32 state, int8 -> int32, or float32 throughout).
//
// For one input row y the update of Sec. 3 (c += w * dh for every event dh of the row) is,
// for each of the three output rows o = y+1-ky the row can influence, a contraction
//     D_ky[x_out][c_out] = sum_{kx, c_in} X[x_out - 1 + kx][c_in] * W[ky][kx][c_in][c_out]
// over the flattened index k = kx * C_in + c_in, for which the operand A[x_out][k] is simply
// the row read as one long vector starting at position x_out - 1.
//
// A workgroup owns a tile of x_out positions and a chunk of output channels for all three ky.
//   * The needed stretch of the input row goes to LDS once.  While it is loaded, every 16-byte
//     cell (position, channel chunk) that holds a non-zero sets a bit; from these bits each wave
//     ballots the list of K-steps whose A fragment is not entirely zero and then visits only
//     those: a stretch of the row without events costs no weight fetch and no matrix
//     instruction (zero values are not events, Sec. 1).
//   * Weights come straight from global memory in the fragment layout (packed once on the host).
//   * The retained rows of c (rows y-1 and y of the rolling buffer) are fetched at the start,
//     straight into the accumulators; row y+1 starts there from the bias.  Epilogue: the row that is now final (y-1; also y
//     when y is the last row of the sample) is activated, rounded to the event type and emitted
//     -- through a fused 2x2 max-pool when one follows -- and forgotten; the others go back to
//     the rolling buffer.
#include "idf.h"
#include "idf_kernels.h"
#include <algorithm>

namespace idf {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

struct TraitsBf16 {
    static constexpr bool kEvents = false;
    static constexpr int kOcc = 3;           // waves per SIMD the batch kernel is compiled for (168 registers)
    static constexpr int kDepth = 3;         // K-steps whose operands are in flight: three waves hide more than six steps did for two
    static constexpr int VL = 8;             // elements per 16-byte lane fragment
    static constexpr int EB = 2;             // bytes per element
    using acc_t = f32x16; using st_t = float; using ev_t = uint16_t;
    static __device__ __forceinline__ acc_t mfma(const i32x4 &a, const i32x4 &b, const acc_t &c)
    {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ bool cell_nonzero(const i32x4 &v)
    {   // bf16 zero is +0 or -0
        return ((v.x | v.y | v.z | v.w) & 0x7fff7fff) != 0;
    }
    static __device__ __forceinline__ int count_nonzero(const i32x4 &v)
    {   // adding 0x7fff to the 15 magnitude bits of a half carries into its top bit unless they are all zero
        int n = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) n += __builtin_popcount((((uint32_t)v[i] & 0x7fff7fffu) + 0x7fff7fffu) & 0x80008000u);
        return n;
    }
    static __device__ __forceinline__ st_t activate(st_t c, int act, int, int) { return act == IDF_ACT_NONE ? c : fmaxf(c, 0.f); }
    static __device__ __forceinline__ ev_t to_ev(st_t h)
    {
        return __builtin_bit_cast(ev_t, (__bf16)h);     // round to nearest, ties to even (one conversion instruction here)
    }
    static __device__ __forceinline__ st_t ev_val(ev_t v) { return __uint_as_float((uint32_t)v << 16); }
    static __device__ __forceinline__ bool ev_nonzero(ev_t v) { return (v & 0x7fffu) != 0; }
    static __device__ __forceinline__ uint32_t bits(ev_t v) { return v; }
    static __device__ __forceinline__ ev_t from_bits(uint32_t u) { return (ev_t)u; }
};

struct TraitsI8 {
    static constexpr bool kEvents = true;    // sparse tiles take the event-list path on the vector units
    static constexpr int kOcc = 2;           // three gain nothing where a launch is one short round of workgroups
    static constexpr int kDepth = 3;           // measured against 4 and 6 on the event workload
    static constexpr int VL = 16;
    static constexpr int EB = 1;
    using acc_t = i32x16; using st_t = int32_t; using ev_t = int8_t;
    static __device__ __forceinline__ acc_t mfma(const i32x4 &a, const i32x4 &b, const acc_t &c)
    {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ bool cell_nonzero(const i32x4 &v) { return (v.x | v.y | v.z | v.w) != 0; }
    static __device__ __forceinline__ int count_nonzero(const i32x4 &v)
    {
        int n = 0;          // per byte: the low seven bits carry into the top bit, or the top bit is set already
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t u = (uint32_t)v[i];
            n += __builtin_popcount((((u & 0x7f7f7f7fu) + 0x7f7f7f7fu) | u) & 0x80808080u);
        }
        return n;
    }
    static __device__ __forceinline__ st_t activate(st_t c, int act, int shr, int hi)
    {
        if (act == IDF_ACT_NONE) return c;
        st_t r = c > 0 ? c : 0;
        if (act == IDF_ACT_RELU_SHR_CLAMP) { r >>= shr; r = r > hi ? hi : r; }
        return r;
    }
    static __device__ __forceinline__ ev_t to_ev(st_t h) { return (ev_t)h; }
    static __device__ __forceinline__ st_t ev_val(ev_t v) { return v; }
    static __device__ __forceinline__ bool ev_nonzero(ev_t v) { return v != 0; }
    static __device__ __forceinline__ uint32_t bits(ev_t v) { return (uint32_t)(uint8_t)v; }
    static __device__ __forceinline__ ev_t from_bits(uint32_t u) { return (ev_t)(uint8_t)u; }
};

// float32 events, weights and state: the 16-byte fragment of a lane holds four k, served by four
// 32x32x2 matrix instructions (instruction i pairs element i of the two half-waves' fragments;
// which two k share an instruction does not matter to the sum).
struct TraitsF32 {
    static constexpr bool kEvents = false;
    static constexpr int kOcc = 2;
    static constexpr int kDepth = 3;         // a step is twelve long matrix instructions here: little to hide
    static constexpr int VL = 4;
    static constexpr int EB = 4;
    using acc_t = f32x16; using st_t = float; using ev_t = float;
    static __device__ __forceinline__ acc_t mfma(const i32x4 &a, const i32x4 &b, acc_t c)
    {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(__int_as_float(a[i]), __int_as_float(b[i]), c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ bool cell_nonzero(const i32x4 &v)
    {   // zero is +0 or -0
        return ((v.x | v.y | v.z | v.w) & 0x7fffffff) != 0;
    }
    static __device__ __forceinline__ int count_nonzero(const i32x4 &v)
    {
        int n = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) n += (v[i] & 0x7fffffff) != 0;
        return n;
    }
    static __device__ __forceinline__ st_t activate(st_t c, int act, int, int) { return act == IDF_ACT_NONE ? c : fmaxf(c, 0.f); }
    static __device__ __forceinline__ ev_t to_ev(st_t h) { return h; }
    static __device__ __forceinline__ st_t ev_val(ev_t v) { return v; }
    static __device__ __forceinline__ bool ev_nonzero(ev_t v) { return v != 0.f; }
    static __device__ __forceinline__ uint32_t bits(ev_t v) { return __float_as_uint(v); }
    static __device__ __forceinline__ ev_t from_bits(uint32_t u) { return __uint_as_float(u); }
};

// A 4-byte cell at a byte offset from a base every lane shares.
template <class P> __device__ __forceinline__ P *at4(P *base, uint32_t byte_off)
{
    return (P *)((const char *)base + byte_off);      // plain pointer arithmetic: the address space stays known
}

constexpr int kMaxPos = 128 + 2;                 // positions of the widest tile plus halo
constexpr int kEvCap = 256;                      // events (tile and halo) the event path takes at most

// LDS the event path needs behind the stretch / staging area: offsets and counts per position, the
// packed event list, and the sums it hands to the accumulators.
// and the tile's share of the layer's weights (three words per input channel and output channel).
constexpr size_t event_lds_bytes(int mt, int nc, int c_in) { return (size_t)(2 * (mt + 4) + kEvCap + 3 * mt * nc + 3 * c_in * nc) * 4; }
constexpr int kNzWords = (kMaxPos + 31) / 32 + 1;

// DBL: a step may take two consecutive input rows (MfmaStep::dbl): the second is worked on by the
// same workgroup straight after the first, with the two rows of c that the first leaves unfinished
// staying in the accumulators (they move up by one tap row) instead of going to the rolling buffer
// and back -- every sum is formed in the same order as by two steps, so the values are the same.
template <class T, int WM, int WN, bool COUNT, bool EV, bool DBL = false>
__device__ __forceinline__ void conv3x3_row(const MfmaStep &a, const StreamSel &sel, const int bx, const int si,
                                            const uint32_t a_at, const uint32_t sel_at)
{
    using acc_t = typename T::acc_t; using st_t = typename T::st_t; using ev_t = typename T::ev_t;
    constexpr int VL = T::VL, EB = T::EB, KI = 2 * VL;
    constexpr int MT = 32 * WM, NC = 32 * WN, NT = 64 * WM * WN;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ uint32_t nz[64][kNzWords];          // per channel chunk: positions with a non-zero cell
    __shared__ unsigned long long red[2][WM * WN];
    __shared__ unsigned int red_ev[WM * WN];       // events of the tile and its halo, per wave (event path)

    // Every argument the kernel uses is asked for here, in one batch of scalar loads with one
    // wait: left to first use, the loads end up behind conditions and cost one memory round
    // trip each, one after the other.
    // Before that batch, one word of every 64-byte line of this step's arguments (they lie a_at
    // bytes into the kernel-argument segment, the stream selection sel_at bytes) is asked for and
    // never looked at: the compiler fetches some arguments again later rather than keep them in
    // registers, and a launch's argument segment is new memory to every scalar cache -- with the
    // lines all requested in the first round, those later fetches find them there instead of
    // paying one miss after the other.  (The register the words land in stays reserved until the
    // batch's own wait has passed: nothing else may be written to it while they are in flight.)
    uint32_t line_touch;
    {
        typedef const __attribute__((address_space(4))) char *karg_ptr;
        const karg_ptr ka = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr() + a_at;
        const karg_ptr ks = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr() + sel_at;
        static_assert(sizeof(MfmaStep) > 0x180 && sizeof(MfmaStep) <= 0x1c0, "one request per 64-byte line of a step's arguments");
        asm volatile("s_load_dword %0, %1, 0x0\n\ts_load_dword %0, %1, 0x40\n\ts_load_dword %0, %1, 0x80\n\t"
                     "s_load_dword %0, %1, 0xc0\n\ts_load_dword %0, %1, 0x100\n\ts_load_dword %0, %1, 0x140\n\t"
                     "s_load_dword %0, %1, 0x180\n\ts_load_dword %0, %1, %3\n\ts_load_dword %0, %2, 0x0"
                     : "=&s"(line_touch)
                     : "s"(ka), "s"(ks), "n"(sizeof(MfmaStep) - 4));
    }
    asm volatile("" ::"s"(a.w), "s"(a.c_in), "s"(a.c_out), "s"(a.c_out_pad), "s"(a.c_in_rcp), "s"(a.chunks_rcp), "s"(a.act), "s"(a.shr),
                 "s"(a.clamp_hi), "s"(a.x_lo), "s"(a.x_hi), "s"(a.skip_clear_tiles), "s"(a.layer), "s"(a.pool_layer), "s"(a.n_layers), "s"(a.taps_y), "s"(a.in_by_position),
                 "s"(a.to_output), "s"(a.in), "s"(a.in_stream_stride), "s"(a.in_row_off), "s"(a.ring),
                 "s"(a.ring_stream_stride), "s"(a.held), "s"(a.held_stream_stride), "s"(a.dst), "s"(a.dst_stream_stride),
                 "s"(a.wfrag), "s"(a.bias), "s"(a.stats));
    asm volatile("" ::"s"(a.t[0].valid), "s"(a.t[0].fresh), "s"(a.t[0].emit), "s"(a.t[0].store_held), "s"(a.t[0].ring_slot),
                 "s"(a.t[0].dst_slot), "s"(a.t[1].valid), "s"(a.t[1].fresh), "s"(a.t[1].emit), "s"(a.t[1].store_held),
                 "s"(a.t[1].ring_slot), "s"(a.t[1].dst_slot), "s"(a.t[2].valid), "s"(a.t[2].fresh), "s"(a.t[2].emit),
                 "s"(a.t[2].store_held), "s"(a.t[2].ring_slot), "s"(a.t[2].dst_slot), "s"(sel.n), "s"(sel.base), "s"(sel.pos0));
    asm volatile("" ::"s"(line_touch));
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int stream = sel_stream(sel, si);
    const int n_co_chunks = (a.c_out + NC - 1) / NC;
    const int x_tile = bx / n_co_chunks, co_chunk = bx - x_tile * n_co_chunks;
    const int x0 = x_tile * MT, co0 = co_chunk * NC;
    if (x0 >= a.w) return;                         // a launch of several steps is as deep as its largest
    // a pixel segment in the middle of a row: tiles it cannot reach are left alone
    if (a.skip_clear_tiles && (x0 + MT < a.x_lo || x0 > a.x_hi)) return;
    const int W = a.w, C_in = a.c_in, C_out = a.c_out;
    const int chunks = C_in / VL;                  // 16-byte cells per position
    const int xs_stride = C_in * EB + 16;          // bytes per position in LDS (padded against bank conflicts)

    // Order of the global loads: the hardware counts outstanding loads in issue order, so what
    // is needed first is requested first -- the row stretch, then the retained state -- and
    // waiting for the stretch leaves the state in flight.  The first weights are asked for only
    // once the stretch has left its registers, and the pool's held row only in the epilogue:
    // with fewer values alive at once, more waves fit a SIMD, which hides more than the earlier
    // requests did.
    const int row_lane = (lane >> 5) * 4;          // D layout: row = 8*i + (lane/32)*4 + j, col = lane%32
    const int xo_base = x0 + wm * 32 + row_lane;
    const int co = co0 + wn * 32 + (lane & 31);
    const bool co_ok = co < C_out;
    // Addresses are clamped into the row instead of predicated per lane: the loads then sit in
    // straight-line code; lanes outside the tile simply never store.
    const int co_c = co_ok ? co : C_out - 1;
    const bool small_c = C_in < VL;                // first layers: 1..4 input channels
    const int64_t in_idx = a.in_by_position ? (int64_t)(sel.pos0 + si) : (int64_t)stream;
    const unsigned char *in_base = (const unsigned char *)a.in + in_idx * a.in_stream_stride * EB;
    acc_t acc[3];
    ev_t hprev[16];                                   // activations of an even row of a pool pair whose partner follows in this launch
#pragma unroll
    for (int q = 0; q < 16; ++q) hprev[q] = 0;
    const int n_sub = DBL ? (a.dbl ? 2 : 1) : 1;
#pragma unroll
    for (int sub = 0; sub < (DBL ? 2 : 1); ++sub) {           // two copies of the body: each is straight-line code for the compiler
    if (sub >= n_sub) break;
    const bool second = DBL && sub > 0;
    auto tap = [&](int ky) -> const MfmaTap & { return second ? a.t2[ky] : a.t[ky]; };
    const unsigned char *in_row = in_base + (second ? a.in_row_off2 : a.in_row_off) * EB;
    if (second) lds_barrier();                     // the first row's stretch, bits and staged rows are done with
    for (int i = tid; i < chunks * kNzWords; i += NT) nz[i / kNzWords][i % kNzWords] = 0;

    // ---- (1) input row stretch [x0-1, x0+MT+1): first batch of 16-byte cells ------------------
    constexpr int kBatch = 9;                      // cells per lane per batch (one batch for C_in <= 256 at 64 positions)
    const int cells = small_c ? 0 : (MT + 2) * chunks;
    i32x4 tv[kBatch];
    auto tile_issue = [&](int base) {
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            if (base + b * NT >= cells) break;         // the same for every lane: narrow layers ask for less
            int i = base + b * NT + tid;
            i = i < cells ? i : cells - 1;
            const int p = a.chunks_rcp ? (int)__umulhi((unsigned)i, a.chunks_rcp) : i, c = i - p * chunks;   // i / chunks
            int x = x0 - 1 + p;
            x = x < a.x_lo ? a.x_lo : (x >= a.x_hi ? a.x_hi - 1 : x);
            tv[b] = *at4(reinterpret_cast<const i32x4 *>(in_row), (uint32_t)((x * C_in + c * VL) * EB));
        }
    };
    if (cells > 0) tile_issue(0);

    // ---- (2) retained rows of c, the bias ------------------------------------------------------
    // This lane's 16 cells of a row [W][C_out]: element offsets (clamped into the row, so loads
    // need no predicate) and which of them exist.  A wave whose cells all exist -- every wave
    // when W is a multiple of 32 and C_out a multiple of the chunk -- stores without predicates.
    // (kept as 32-bit byte offsets of 4-byte cells: with the row's base in scalar registers an
    // access is then "scalar base + lane offset", no 64-bit arithmetic per cell)
    uint32_t roff[16];
    unsigned int vmask = 0;
    auto cell_offsets = [&](int xo_first) {
        vmask = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int xo = xo_first + 8 * i + j;
                roff[i * 4 + j] = (uint32_t)(((xo < W ? xo : W - 1) * C_out + co_c) * 4);
                vmask |= (co_ok && xo < W) ? 1u << (i * 4 + j) : 0u;
            }
    };
    cell_offsets(xo_base);
    const bool wave_full = __ballot(vmask != 0xffffu) == 0ull;
    const st_t bias_v = a.bias ? ((const st_t *)a.bias)[co_c] : (st_t)0;
    st_t *ring = (st_t *)a.ring + (int64_t)stream * a.ring_stream_stride;
    // They are loaded straight into the accumulators (a row touched for the first time starts
    // from the bias there): the contraction then adds on top and the epilogue has nothing to add.
    if (!second) {
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const st_t start = a.t[ky].valid ? bias_v : (st_t)0;
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[ky][q] = start;
            if (a.t[ky].valid && !a.t[ky].fresh) {
                const st_t *rrow = ring + (int64_t)a.t[ky].ring_slot * W * C_out;
#pragma unroll
                for (int q = 0; q < 16; ++q) acc[ky][q] = *at4(rrow, roff[q]);
            }
        }
    } else {
        // rows y and y+1 are in the accumulators already: one tap row up; row y+2 starts from the bias
        acc[2] = acc[1];
        acc[1] = acc[0];
        const st_t start = a.t2[0].valid ? bias_v : (st_t)0;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[0][q] = start;
    }
    ev_t *held = (ev_t *)a.held + (int64_t)stream * a.held_stream_stride;

    // ---- (3) weight fragments: addressing -------------------------------------------------------
    const int KT = 3 * C_in;
    const int steps = (KT + KI - 1) / KI;
    const int hlf = lane >> 5, r = wm * 32 + (lane & 31);
    // weights: the three ky planes as scalar bases, this lane's fragment as a 32-bit byte offset
    const uint32_t w_lane = (uint32_t)((hlf * a.c_out_pad + co0 + wn * 32 + (lane & 31)) * 16);
    const uint32_t w_step = (uint32_t)(2 * a.c_out_pad * 16);       // bytes per K-step
    const i32x4 *w_plane[3];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
        w_plane[ky] = reinterpret_cast<const i32x4 *>((const unsigned char *)a.wfrag + (int64_t)ky * steps * w_step);
    constexpr int kDepth = T::kDepth;                                // K-steps in flight
    i32x4 aq[kDepth], bq[kDepth][3];
    auto fetch_b = [&](int d, int sn) {
        const uint32_t off = w_lane + (uint32_t)sn * w_step;
        bq[d][0] = *at4(w_plane[0], off);
        bq[d][1] = *at4(w_plane[1], off);
        bq[d][2] = *at4(w_plane[2], off);
    };

    // ---- stretch -> LDS, with occupancy bits and the counters ---------------------------------
    lds_barrier();                               // occupancy bits are cleared
    {
        const bool count = co_chunk == 0 && a.stats;
        const bool weigh = EV && a.ev_limit > 0;   // the tile's events decide which way it goes
        unsigned int ev = 0, taps = 0;               // per lane: a few cells
        unsigned int ev_all = 0;                     // halo included
        if (!small_c) {
            for (int base = 0; base < cells; base += NT * kBatch) {
                if (base > 0) tile_issue(base);
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    const int i = base + b * NT + tid;
                    if (i >= cells) continue;
                    const int p = a.chunks_rcp ? (int)__umulhi((unsigned)i, a.chunks_rcp) : i, c = i - p * chunks;
                    const int x = x0 - 1 + p;
                    if (x < a.x_lo || x >= a.x_hi) tv[b] = i32x4{0, 0, 0, 0};
                    *reinterpret_cast<i32x4 *>(smem + p * xs_stride + c * 16) = tv[b];
                    if (T::cell_nonzero(tv[b])) {
                        atomicOr(&nz[c][p >> 5], 1u << (p & 31));
                        if (weigh || (count && p >= 1 && p <= MT)) {
                            const int n = T::count_nonzero(tv[b]);
                            ev_all += n;
                            if (count && p >= 1 && p <= MT) {
                                ev += n;
                                taps += n * (3 - (x == 0) - (x == W - 1));
                            }
                        }
                    }
                }
            }
        } else {
            // the stretch is kept as one flat vector: A[x_out][k] is element (x_out - x0) * C_in + k of it
            const ev_t *in_e = reinterpret_cast<const ev_t *>(in_row);
            ev_t *xs_e = reinterpret_cast<ev_t *>(smem);
            const int elems = (MT + 2) * C_in;
            for (int i = tid; i < elems; i += NT) {
                const int p = i / C_in;
                const int x = x0 - 1 + p;
                ev_t v = 0;
                if (x >= a.x_lo && x < a.x_hi) v = *at4(in_e, (uint32_t)((x * C_in + (i - p * C_in)) * EB));
                xs_e[i] = v;
                if (T::ev_nonzero(v)) {
                    ev_all += 1;
                    if (count && p >= 1 && p <= MT) {
                        ev += 1;
                        taps += 3 - (x == 0) - (x == W - 1);
                    }
                }
            }
        }
        if (count) {
            for (int off = 32; off > 0; off >>= 1) { ev += __shfl_down(ev, off); taps += __shfl_down(taps, off); }
            if (lane == 0) { red[0][wave] = ev; red[1][wave] = taps; }
        }
        if (weigh) {
            for (int off = 32; off > 0; off >>= 1) ev_all += __shfl_down(ev_all, off);
            if (lane == 0) red_ev[wave] = ev_all;
        }
        if (!small_c && tid == 0) *reinterpret_cast<i32x4 *>(smem + C_in * EB) = i32x4{0, 0, 0, 0};      // the padding behind position 0: a cell of zeros
        lds_barrier();
        if (count && tid == 0) {
            unsigned long long e = 0, t = 0;
            for (int wv = 0; wv < WM * WN; ++wv) { e += red[0][wv]; t += red[1][wv]; }
            unsigned long long *dst = a.stats + ((int64_t)stream * a.n_layers + a.layer) * 2;
            if (e) atomicAdd(dst, e);
            if (t) atomicAdd(dst + 1, t * (unsigned long long)((second ? a.taps_y2 : a.taps_y) * C_out));
        }
    }

    // weights of the first K-steps, before it is known which steps are live
#pragma unroll
    for (int d = 0; d < kDepth; ++d) fetch_b(d, d < steps ? d : steps - 1);

    // ---- sparse tiles: the event-list path ------------------------------------------------------
    // Zero values are not events (Sec. 1): where a tile and its halo hold few of them, the update is
    // done event by event on the vector units instead of as a contraction that multiplies the zeros.
    //   1. Every position's non-zero values are counted (one lane per position), an exclusive prefix
    //      sum over the positions gives each its place in a packed list, and the events (channel,
    //      value) are written there position by position: a compressed row.
    //   2. If the list is short enough (the host's cost model says up to how many events the vector
    //      units are the faster way), lanes = output channels take the tile's output positions in
    //      turn; for a position the events of its three input positions lie one after the other in
    //      the list; each event costs one weight word (the three ky taps of its (kx, channel) for
    //      this lane's output channel) and three multiply-adds.  The sums go to the matrix path's
    //      accumulators through LDS, and everything after is common.
    bool use_events = false;
    if constexpr (EV) {
        if (a.ev_limit > 0) {
            const size_t front = (size_t)(MT + 2) * (small_c ? C_in * EB : xs_stride), stg = (size_t)MT * NC * EB;
            int32_t *ev_cnt = reinterpret_cast<int32_t *>(smem + (((front > stg ? front : stg) + 15) & ~(size_t)15));
            int32_t *ev_off = ev_cnt + (MT + 4);
            uint32_t *ev_list = reinterpret_cast<uint32_t *>(ev_off + (MT + 4));
            int32_t *dsum = reinterpret_cast<int32_t *>(ev_list + kEvCap);
            uint32_t *wlds = reinterpret_cast<uint32_t *>(dsum + 3 * MT * NC);      // [kx][c_in][NC]
            const ev_t *xs_flat = reinterpret_cast<const ev_t *>(smem);
            // visits every non-zero value of stretch position p in channel order
            auto for_events = [&](int p, auto &&f) {
                if (small_c) {
                    for (int ci = 0; ci < C_in; ++ci) {
                        const ev_t v = xs_flat[p * C_in + ci];
                        if (T::ev_nonzero(v)) f(ci, v);
                    }
                } else {
                    for (int c = 0; c < chunks; ++c) {
                        if (!(nz[c][p >> 5] >> (p & 31) & 1u)) continue;
                        const ev_t *cell = reinterpret_cast<const ev_t *>(smem + p * xs_stride + c * 16);
                        for (int e = 0; e < VL; ++e)
                            if (T::ev_nonzero(cell[e])) f(c * VL + e, cell[e]);
                    }
                }
            };
            unsigned int n_ev = 0;
            for (int wv = 0; wv < WM * WN; ++wv) n_ev += red_ev[wv];
            use_events = n_ev <= (unsigned)a.ev_limit && n_ev <= (unsigned)kEvCap;
            if (use_events && n_ev > 0) {
                // the tile's share of the weights, asked for first: on its way while the list is made
                {
                    const uint32_t *wsrc = reinterpret_cast<const uint32_t *>(a.w_ev) + co0;
                    for (int i = tid; i < 3 * C_in * NC; i += NT) {
                        const int row = i / NC, col = i - row * NC;
                        wlds[i] = wsrc[(size_t)row * a.c_out_pad + col];
                    }
                }
                int my_cnt = 0;
                if (tid < MT + 2) {
                    for_events(tid, [&](int, ev_t) { ++my_cnt; });
                    ev_cnt[tid] = my_cnt;
                }
                lds_barrier();
                if (tid <= MT + 2) {                 // exclusive prefix: where position tid's events begin (entry MT+2: the total)
                    int o = 0;
                    for (int q = 0; q < tid; ++q) o += ev_cnt[q];
                    ev_off[tid] = o;
                }
                lds_barrier();
            }
            if (use_events && n_ev > 0) {
                if (tid < MT + 2) {
                    int at = ev_off[tid];
                    for_events(tid, [&](int ci, ev_t v) { ev_list[at++] = ((uint32_t)ci << 8) | (T::bits(v) & 0xffu); });
                }
                lds_barrier();
                constexpr int PG = NT / NC;              // output positions worked on side by side
                const int co_l = tid % NC, pg = tid / NC;
                const uint32_t *wev = wlds + co_l;
                unsigned long long visits = 0;
                for (int r = pg; r < MT; r += PG) {
                    const int i0 = ev_off[r], i1 = ev_off[r + 1], i2 = ev_off[r + 2], i3 = ev_off[r + 3];
                    int32_t d0 = 0, d1 = 0, d2 = 0;
                    for (int idx = i0; idx < i3; idx += 4) {
                        uint32_t wv[4];
                        int32_t vv[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {        // the four weight words are asked for before the first is used
                            const int id = idx + u;
                            const bool ok = id < i3;
                            const uint32_t e = ev_list[ok ? id : i0];
                            const int kx = (id >= i1) + (id >= i2);
                            const int ci = (int)(e >> 8);
                            vv[u] = ok ? (int32_t)(int8_t)(e & 0xffu) : 0;
                            wv[u] = wev[(ok ? kx * C_in + ci : 0) * NC];
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            d0 += vv[u] * (int32_t)(int8_t)(wv[u] & 0xffu);
                            d1 += vv[u] * (int32_t)(int8_t)((wv[u] >> 8) & 0xffu);
                            d2 += vv[u] * (int32_t)(int8_t)((wv[u] >> 16) & 0xffu);
                        }
                    }
                    dsum[(0 * MT + r) * NC + co_l] = d0;
                    dsum[(1 * MT + r) * NC + co_l] = d1;
                    dsum[(2 * MT + r) * NC + co_l] = d2;
                    visits += (unsigned long long)(i3 - i0);
                }
                if (COUNT && a.issued && co_l == 0 && visits)
                    atomicAdd(a.issued + (int64_t)stream * a.n_layers + a.layer, visits * (3ull * NC));
                lds_barrier();
                const int dcol = wn * 32 + (lane & 31), drow = wm * 32 + row_lane;
#pragma unroll
                for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[ky][i * 4 + j] += (st_t)dsum[(ky * MT + drow + 8 * i + j) * NC + dcol];
            }
        }
    }

    // ---- which K-steps have anything in them for this wave's 32 positions -------------------
    unsigned long long live;
    if (!use_events) {
        bool occ = small_c && lane < steps;          // few channels: every step is visited
        if (!small_c && lane < steps) {
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                const int k0 = lane * KI + h2 * VL;
                if (k0 < KT) {
                    const int kx = k0 / C_in, c = (k0 - kx * C_in) / VL;
                    const int start = wm * 32 + kx;               // first tile position of the window
                    const uint32_t lo = nz[c][start >> 5], hi = nz[c][(start >> 5) + 1];
                    const uint32_t win = (uint32_t)((((unsigned long long)hi << 32) | lo) >> (start & 31));
                    occ |= win != 0;
                }
            }
        }
        live = __ballot(occ);
        // what the matrix instructions of this wave will multiply, zeros inside a live step included
        if (COUNT && a.issued && lane == 0 && live)
            atomicAdd(a.issued + (int64_t)stream * a.n_layers + a.layer,
                      (unsigned long long)__builtin_popcountll(live) * (3ull * 32 * 32 * KI));
    }

    else live = 0;

    // ---- contraction over the live K-steps ----------------------------------------------------
    if (use_events) {
        // done above, event by event
    } else if (small_c) {
        // first layers: K = 3*C_in <= 12, one or two steps (all prefetched); the fragment is gathered
        // element by element
        const ev_t *xs_e = reinterpret_cast<const ev_t *>(smem) + r * C_in;
#pragma unroll
        for (int sn = 0; sn < (12 + KI - 1) / KI; ++sn) {
            if (sn >= steps) break;
            const int k0 = sn * KI + hlf * VL;
            ev_t e[VL];
#pragma unroll
            for (int q = 0; q < VL; ++q) e[q] = k0 + q < KT ? xs_e[k0 + q] : (ev_t)0;
            i32x4 av;
            __builtin_memcpy(&av, e, 16);
            acc[0] = T::mfma(av, bq[sn][0], acc[0]);
            acc[1] = T::mfma(av, bq[sn][1], acc[1]);
            acc[2] = T::mfma(av, bq[sn][2], acc[2]);
        }
    } else {
        // Software pipeline over the live steps, kDepth steps deep.  Every slot issues its loads
        // unconditionally (past the end the last live step is simply fetched again), so the
        // loop body is straight-line code and each slot waits for exactly its own operands.
        const int n_live = __builtin_popcountll(live);
        int s_last = 0;
        bool any_left = true;
        auto next_step = [&]() {
            const int f = __builtin_ffsll((long long)live);           // 0 when nothing is left
            any_left = f != 0;
            const int sn = f ? f - 1 : s_last;
            s_last = sn;
            live &= live - 1;
            return sn;
        };
        auto fetch_a = [&](int d, int sn) {
            const int k0 = sn * KI + hlf * VL;
            const int kx = (int)__umulhi((unsigned)k0, a.c_in_rcp);   // k0 / C_in
            const int ci = k0 - kx * C_in;
            // half a step of padding at the end of K, and slots past the last live step: these read the cell of zeros
            // behind position 0 (no select after the read, so nothing waits for it before the slot's turn comes)
            const bool ok = any_left && k0 < KT;
            aq[d] = *reinterpret_cast<const i32x4 *>(smem + (ok ? (r + kx) * xs_stride + ci * EB : C_in * EB));
        };
        if (n_live > 0) {
            int sn0[kDepth];
            bool guessed = true;
#pragma unroll
            for (int d = 0; d < kDepth; ++d) {
                sn0[d] = next_step();
                fetch_a(d, sn0[d]);
                guessed &= sn0[d] == (d < steps ? d : steps - 1);
            }
            // a wrong guess: all slots again, in slot order -- whichever way the loop is entered, the youngest requests
            // are then slot 0's, 1's, ... in turn, and each slot's wait inside the loop can leave the others in flight
            if (!guessed) {
#pragma unroll
                for (int d = 0; d < kDepth; ++d) fetch_b(d, sn0[d]);
            }
            for (int it = 0; it < n_live; it += kDepth) {
#pragma unroll
                for (int d = 0; d < kDepth; ++d) {
                    // no branch around these: past the last live step the slot multiplies zeros, and the loop body stays
                    // one straight line in which every slot's wait leaves the younger slots' requests in flight
                    acc[0] = T::mfma(aq[d], bq[d][0], acc[0]);
                    acc[1] = T::mfma(aq[d], bq[d][1], acc[1]);
                    acc[2] = T::mfma(aq[d], bq[d][2], acc[2]);
                    const int sn = next_step();
                    fetch_a(d, sn);
                    fetch_b(d, sn);
                    __builtin_amdgcn_sched_barrier(0);      // the slots stay in this order: requests go out right behind their slot's matrix instructions
                }
            }
        }
    }

    // ---- epilogue -----------------------------------------------------------------------------
    // Rows of c go back to the ring straight from the accumulator layout (32 lanes x 4 bytes = one
    // full 128-byte line per row of the tile).  Event-type rows (1 or 2 bytes per value) would be
    // partial-line writes from that layout, so they are staged in LDS as [position][channel] and
    // leave as 16-byte chunks that tile whole lines.
    if (T::kOcc > 2) {
        // The offsets are worked out again rather than kept: sixteen registers held across the
        // contraction would be spilled to memory by every lane at three waves per SIMD.  (The
        // empty statement hides from the compiler that it has seen this value before.)
        int xo_again = xo_base;
        asm volatile("" : "+v"(xo_again));
        cell_offsets(xo_again);
    }
    ev_t *stage = reinterpret_cast<ev_t *>(smem);
    bool stage_free = false;                          // the stretch in LDS may still be read by slower waves
    auto flush = [&](ev_t *grow, int row_w, int p0, int npos) {
        // grow: the row [x][C_out] in global memory; positions p0 .. p0+npos-1 of it are staged
        lds_barrier();
        constexpr int kPer = 16 / EB;                 // channels per 16-byte chunk
        constexpr int kCpp = NC / kPer;               // chunks per position
        for (int i = tid; i < npos * kCpp; i += NT) {
            const int p = i / kCpp, k = i - p * kCpp;
            const int x = p0 + p, cch = co0 + k * kPer;
            if (x < row_w && cch < C_out)
                *at4(reinterpret_cast<i32x4 *>(grow), (uint32_t)((x * C_out + cch) * EB)) =
                    *reinterpret_cast<const i32x4 *>(stage + p * NC + k * kPer);
        }
        lds_barrier();
    };
    const int col = wn * 32 + (lane & 31);            // channel within the chunk
    const int prow = wm * 32 + row_lane;              // first of this lane's positions within the tile
    uint32_t heldv[16];                               // the pool's held row: one register each, nothing to pack
    {
        const bool need = tap(2).valid && tap(2).emit == kEmitPoolHeld;   // only row y-1 can pair with the held row
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            heldv[q] = 0;
            if (need) heldv[q] = T::bits(*at4(held, roff[q] / (4 / EB)));
        }
    }
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) {
        const int ky = 2 - kk;                        // row y-1 first
        const MfmaTap &t = tap(ky);
        if (!t.valid) continue;
        if (DBL && t.emit == kEmitKeep) continue;     // stays in the accumulators for the second row
        st_t c[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) c[q] = acc[ky][q];
        if (t.emit == kEmitNone) {
            st_t *rrow = ring + (int64_t)t.ring_slot * W * C_out;
            if (wave_full) {
#pragma unroll
                for (int q = 0; q < 16; ++q) *at4(rrow, roff[q]) = c[q];
            } else {
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if (vmask >> q & 1u) *at4(rrow, roff[q]) = c[q];
            }
            continue;
        }
        ev_t e[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) e[q] = T::to_ev(T::activate(c[q], a.act, a.shr, a.clamp_hi));
        if (a.pool_layer >= 0 && a.stats) {          // what the fused pool receives counts as its events
            unsigned int n = 0;
#pragma unroll
            for (int q = 0; q < 16; ++q) n += ((vmask >> q & 1u) && T::ev_nonzero(e[q])) ? 1u : 0u;
            for (int off = 32; off > 0; off >>= 1) n += __shfl_down(n, off);
            if (lane == 0 && n)
                atomicAdd(a.stats + ((int64_t)stream * a.n_layers + a.pool_layer) * 2, (unsigned long long)n);
        }
        if (t.emit == kEmitDirect && a.to_output) {
            // last layer: 4-byte values, not rounded to the event type
            st_t *orow = (st_t *)a.dst + (int64_t)stream * a.dst_stream_stride + t.dst_slot * W * C_out;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                if (wave_full || (vmask >> q & 1u)) *at4(orow, roff[q]) = T::activate(c[q], a.act, a.shr, a.clamp_hi);
        } else if (t.emit == kEmitDirect || (t.emit == kEmitHold && t.store_held)) {
            if (!stage_free) { lds_barrier(); stage_free = true; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) stage[(prow + 8 * i + j) * NC + col] = e[i * 4 + j];
            ev_t *grow = t.emit == kEmitHold
                             ? held
                             : (ev_t *)a.dst + (int64_t)stream * a.dst_stream_stride + t.dst_slot * W * C_out;
            flush(grow, W, x0, MT);
        }
        if (t.emit == kEmitHold) {
#pragma unroll
            for (int q = 0; q < 16; ++q) hprev[q] = e[q];
        } else if (t.emit == kEmitPoolHeld || t.emit == kEmitPoolReg) {
            // 2x2 max: this row and the even row of the pair, positions 2j and 2j+1 (both in this lane)
            const int Wp = W / 2;
            if (!stage_free && !a.to_output) { lds_barrier(); stage_free = true; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    st_t m = T::ev_val(e[i * 4 + 2 * jj]);
                    const st_t m1 = T::ev_val(e[i * 4 + 2 * jj + 1]);
                    m = m1 > m ? m1 : m;
                    st_t e0, e1;
                    if (t.emit == kEmitPoolHeld) {
                        e0 = T::ev_val(T::from_bits(heldv[i * 4 + 2 * jj]));
                        e1 = T::ev_val(T::from_bits(heldv[i * 4 + 2 * jj + 1]));
                    } else {
                        e0 = T::ev_val(hprev[i * 4 + 2 * jj]);
                        e1 = T::ev_val(hprev[i * 4 + 2 * jj + 1]);
                    }
                    m = e0 > m ? e0 : m;
                    m = e1 > m ? e1 : m;
                    const int pl = ((prow + 8 * i) >> 1) + jj;        // pooled position within the tile
                    if (a.to_output) {
                        const int xp = (x0 >> 1) + pl;
                        if (co_ok && xp < Wp)
                            ((st_t *)a.dst)[(int64_t)stream * a.dst_stream_stride + (t.dst_slot * Wp + xp) * C_out + co] = m;
                    } else {
                        stage[pl * NC + col] = T::to_ev(m);
                    }
                }
            if (!a.to_output)
                flush((ev_t *)a.dst + (int64_t)stream * a.dst_stream_stride + t.dst_slot * Wp * C_out, Wp, x0 >> 1, MT / 2);
        }
    }
    }   // rows of the step
}

template <class T, int WM, int WN, bool COUNT, bool EV>
__global__ void __launch_bounds__(64 * WM * WN, 2) k_conv3x3_mfma(const MfmaStep a, const StreamSel sel)
{
    // tile by tile, the streams of a tile side by side
    conv3x3_row<T, WM, WN, COUNT, EV>(a, sel, blockIdx.z, blockIdx.x, 0, (uint32_t)sizeof(MfmaStep));
}

// Several layers' steps in one launch (each on a row that was complete before the launch).  The grid
// is (stream, tile, step): a workgroup knows its step from its own index, so its arguments arrive in
// one round of scalar loads (a table of first tiles per step cost a second, dependent round: about
// half a microsecond before the first row request of every workgroup).  Steps with fewer tiles than
// the launch's largest leave a few workgroups that return at once.  One tile shape for all steps.
// In dispatch order the streams of a tile lie side by side, then the tiles of a step, then the steps
// with the deepest (longest) first.  Consecutive workgroups go to the eight XCDs in turn: with a
// multiple of eight streams a stream always meets the same XCD, so its row stretch is fetched into one
// L2 for all its channel chunks, a weight fragment is fetched once per XCD and used by that XCD's
// streams close in time, and every step is spread evenly.  (Stream by stream with the tiles inside was
// measured 8 % slower on the VGG-style workload; one contiguous eighth of the order per XCD slower
// still: the steps differ too much in length.)
// (the form that can take two rows per step keeps a pool's even row in registers across the second
// row's contraction: compiled for two waves per SIMD)
template <class T, int WM, int WN, bool COUNT, bool EV, bool DBL = false>
__global__ void __launch_bounds__(64 * WM * WN, DBL ? 2 : T::kOcc) k_conv3x3_mfma_batch(const MfmaBatch b, const StreamSel sel)
{
    conv3x3_row<T, WM, WN, COUNT, EV, DBL>(b.st[blockIdx.z], sel, blockIdx.y, blockIdx.x,
                                           (uint32_t)(offsetof(MfmaBatch, st) + blockIdx.z * sizeof(MfmaStep)), (uint32_t)sizeof(MfmaBatch));
}

template <class T, int WM, int WN>
hipError_t launch_batch_shape(const MfmaBatch &b, const StreamSel &sel, const LaunchCtx &lc)
{
    constexpr int MT = 32 * WM, NC = 32 * WN;
    size_t lds = 0;
    int tiles_max = 0;
    for (int k = 0; k < b.n; ++k) {
        const MfmaStep &a = b.st[k];
        tiles_max = std::max(tiles_max, ((a.w + MT - 1) / MT) * ((a.c_out + NC - 1) / NC));
        lds = std::max(lds, (size_t)(MT + 2) * (a.c_in * T::EB + 16));
        lds = std::max(lds, (size_t)MT * NC * T::EB);
    }
    if (b.n < 1 || tiles_max < 1 || tiles_max > 65535) return hipErrorInvalidValue;      // tiles are the grid's y extent
    const dim3 grid(sel.n, tiles_max, b.n), block(64 * WM * WN);
    if constexpr (T::kEvents) {
        // room for the event path behind a step's stretch / staging area, or no event path for that step; the kernel
        // that carries the event path is a separate one, so a launch without it pays nothing for it
        MfmaBatch bb = b;
        const size_t base = (lds + 15) & ~(size_t)15;
        bool any = false;
        for (int k = 0; k < bb.n; ++k) {
            if (bb.st[k].ev_limit <= 0) continue;
            const size_t need = base + event_lds_bytes(MT, NC, bb.st[k].c_in);
            if (need <= 64 * 1024) { lds = std::max(lds, need); any = true; }
            else bb.st[k].ev_limit = 0;
        }
        if (any) {
            if (b.st[0].issued) return launch(k_conv3x3_mfma_batch<T, WM, WN, true, true>, grid, block, lds, lc, bb, sel);
            return launch(k_conv3x3_mfma_batch<T, WM, WN, false, true>, grid, block, lds, lc, bb, sel);
        }
    }
    bool two_rows = false;                        // some step takes two input rows: the kernel that can
    for (int k = 0; k < b.n; ++k) two_rows = two_rows || b.st[k].dbl;
    if (two_rows) {
        if constexpr (WM == 1) {                  // (the launches that pair rows use tiles of 32 positions only)
            if (b.st[0].issued) return launch(k_conv3x3_mfma_batch<T, WM, WN, true, false, true>, grid, block, lds, lc, b, sel);
            return launch(k_conv3x3_mfma_batch<T, WM, WN, false, false, true>, grid, block, lds, lc, b, sel);
        } else {
            return hipErrorInvalidValue;
        }
    }
    // the variant that adds up what it issues is a kernel of its own: the one that is timed carries none of it
    if (b.st[0].issued) return launch(k_conv3x3_mfma_batch<T, WM, WN, true, false>, grid, block, lds, lc, b, sel);
    return launch(k_conv3x3_mfma_batch<T, WM, WN, false, false>, grid, block, lds, lc, b, sel);
}

template <class T>
hipError_t launch_batch(const MfmaBatch &b, const StreamSel &sel, const LaunchCtx &lc)
{
    switch (b.tile) {
    case kMfmaTile64x64: return launch_batch_shape<T, 2, 2>(b, sel, lc);
    case kMfmaTile64x32: return launch_batch_shape<T, 2, 1>(b, sel, lc);
    case kMfmaTile32x64: return launch_batch_shape<T, 1, 2>(b, sel, lc);
    case kMfmaTile32x32: return launch_batch_shape<T, 1, 1>(b, sel, lc);
    default: return hipErrorInvalidValue;
    }
}

template <class T, int WM, int WN>
hipError_t launch_one(const MfmaStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    constexpr int MT = 32 * WM, NC = 32 * WN;
    const int x_tiles = (a.w + MT - 1) / MT, co_chunks = (a.c_out + NC - 1) / NC;
    size_t lds = (size_t)(MT + 2) * (a.c_in * T::EB + 16);
    const size_t stage = (size_t)MT * NC * T::EB;       // the epilogue reuses the space to stage emitted rows
    if (lds < stage) lds = stage;
    if (x_tiles * co_chunks > 65535) return hipErrorInvalidValue;      // tiles are the grid's z extent
    const dim3 grid(sel.n, 1, x_tiles * co_chunks), block(64 * WM * WN);
    if constexpr (T::kEvents) {
        const size_t with_events = ((lds + 15) & ~(size_t)15) + event_lds_bytes(MT, NC, a.c_in);
        if (a.ev_limit > 0 && with_events <= 64 * 1024) {
            if (a.issued) return launch(k_conv3x3_mfma<T, WM, WN, true, true>, grid, block, with_events, lc, a, sel);
            return launch(k_conv3x3_mfma<T, WM, WN, false, true>, grid, block, with_events, lc, a, sel);
        }
    }
    if (a.issued) return launch(k_conv3x3_mfma<T, WM, WN, true, false>, grid, block, lds, lc, a, sel);
    return launch(k_conv3x3_mfma<T, WM, WN, false, false>, grid, block, lds, lc, a, sel);
}

template <class T> hipError_t launch_prec(const MfmaStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    switch (a.tile) {
    case kMfmaTile64x64: return launch_one<T, 2, 2>(a, sel, lc);
    case kMfmaTile128x32: return launch_one<T, 4, 1>(a, sel, lc);
    case kMfmaTile32x64: return launch_one<T, 1, 2>(a, sel, lc);
    case kMfmaTile32x32: return launch_one<T, 1, 1>(a, sel, lc);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

// Elements of the event type per 16-byte fragment.
int conv3x3_mfma_vl(int prec) { return prec == IDF_PREC_F32 ? 4 : prec == IDF_PREC_BF16 ? 8 : 16; }

bool conv3x3_mfma_eligible(int prec, const Geom &g)
{
    if (prec != IDF_PREC_BF16 && prec != IDF_PREC_I8 && prec != IDF_PREC_F32) return false;
    const int vl = conv3x3_mfma_vl(prec);
    if (g.kind != IDF_CONV || g.k_h != 3 || g.k_w != 3 || g.s_h != 1 || g.s_w != 1 || g.p_h != 1 || g.p_w != 1) return false;
    if (g.h_in < 2 || g.w_in < 2) return false;
    if ((g.c_in % vl != 0 && g.c_in > 4) || g.c_out % 16 != 0) return false;
    const int steps = (3 * g.c_in + 2 * vl - 1) / (2 * vl);
    if (steps > 64 || g.c_in / vl > 64) return false;
    return true;
}

int conv3x3_mfma_tile(const Geom &g, int n_streams)
{
    // wide tiles reuse each weight fragment for more positions; narrow ones give more workgroups
    if (g.c_out <= 32) return g.w_out > 64 ? kMfmaTile128x32 : kMfmaTile32x32;
    const long wg64 = (long)((g.w_out + 63) / 64) * ((g.c_out + 63) / 64) * n_streams;
    if (g.w_out <= 32 || (wg64 < 256 && g.w_out % 64 != 0 && g.w_out % 64 <= 32)) return kMfmaTile32x64;
    return kMfmaTile64x64;
}

namespace {
void tile_shape(int tile, int &wm, int &wn)
{
    wm = tile == kMfmaTile64x64 || tile == kMfmaTile64x32 ? 2 : tile == kMfmaTile128x32 ? 4 : 1;
    wn = tile == kMfmaTile64x64 || tile == kMfmaTile32x64 ? 2 : 1;
}
}  // namespace

int conv3x3_mfma_tiles(int tile, int w, int c_out)
{
    int wm, wn;
    tile_shape(tile, wm, wn);
    return ((w + 32 * wm - 1) / (32 * wm)) * ((c_out + 32 * wn - 1) / (32 * wn));
}

int conv3x3_mfma_batch_resident(int prec, int tile)
{
    int wm, wn;
    tile_shape(tile, wm, wn);
    const int per_simd = prec == IDF_PREC_BF16 ? TraitsBf16::kOcc : prec == IDF_PREC_I8 ? TraitsI8::kOcc : TraitsF32::kOcc;
    return std::max(1, 4 * per_simd / (wm * wn));
}

// Weights [k_h][k_w][c_in][c_out] -> fragment order [ky][k/VL][c_out_pad][VL] with k = kx*c_in + ci,
// zero padded to whole K-steps and to a multiple of 64 output channels.
size_t conv3x3_mfma_pack(int prec, const Geom &g, const void *w_khkwcico, void *out)
{
    const int vl = conv3x3_mfma_vl(prec), eb = 16 / vl;
    const int KT = 3 * g.c_in, steps = (KT + 2 * vl - 1) / (2 * vl), kc = 2 * steps;
    const int cop = (g.c_out + 63) / 64 * 64;
    const size_t frag_bytes = (size_t)3 * kc * cop * 16;
    // int8: behind the fragments the same weights for the event path, [kx][c_in][cop] words holding the taps ky = 0, 1, 2 of
    // (kx, c_in, c_out) in their three low bytes
    const size_t bytes = frag_bytes + (prec == IDF_PREC_I8 ? (size_t)3 * g.c_in * cop * 4 : 0);
    if (!out) return bytes;
    unsigned char *o = (unsigned char *)out;
    const unsigned char *src = (const unsigned char *)w_khkwcico;
    for (size_t i = 0; i < bytes; ++i) o[i] = 0;
    if (prec == IDF_PREC_I8)
        for (int ky = 0; ky < 3; ++ky)
            for (int kx = 0; kx < 3; ++kx)
                for (int ci = 0; ci < g.c_in; ++ci)
                    for (int co = 0; co < g.c_out; ++co)
                        o[frag_bytes + (((size_t)kx * g.c_in + ci) * cop + co) * 4 + ky] = src[(((size_t)ky * 3 + kx) * g.c_in + ci) * g.c_out + co];
    for (int ky = 0; ky < 3; ++ky)
        for (int k = 0; k < KT; ++k) {
            const int kx = k / g.c_in, ci = k % g.c_in;
            for (int co = 0; co < g.c_out; ++co) {
                const size_t s_idx = (((size_t)ky * 3 + kx) * g.c_in + ci) * g.c_out + co;
                const size_t d_idx = (((size_t)ky * kc + k / vl) * cop + co) * vl + k % vl;
                for (int b = 0; b < eb; ++b) o[d_idx * eb + b] = src[s_idx * eb + b];
            }
        }
    return bytes;
}

size_t conv3x3_mfma_event_weights(int prec, const Geom &g)
{
    if (prec != IDF_PREC_I8) return 0;
    const int vl = conv3x3_mfma_vl(prec);
    const int KT = 3 * g.c_in, steps = (KT + 2 * vl - 1) / (2 * vl);
    return (size_t)3 * 2 * steps * ((g.c_out + 63) / 64 * 64) * 16;
}

int conv3x3_mfma_event_cap() { return kEvCap; }

hipError_t launch_conv3x3_mfma_batch(int prec, const MfmaBatch &b, const StreamSel &sel, const LaunchCtx &lc)
{
    if (prec == IDF_PREC_F32) return launch_batch<TraitsF32>(b, sel, lc);
    if (prec == IDF_PREC_BF16) return launch_batch<TraitsBf16>(b, sel, lc);
    if (prec == IDF_PREC_I8) return launch_batch<TraitsI8>(b, sel, lc);
    return hipErrorInvalidValue;
}

hipError_t launch_conv3x3_mfma(int prec, const MfmaStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    if (prec == IDF_PREC_F32) return launch_prec<TraitsF32>(a, sel, lc);
    if (prec == IDF_PREC_BF16) return launch_prec<TraitsBf16>(a, sel, lc);
    if (prec == IDF_PREC_I8) return launch_prec<TraitsI8>(a, sel, lc);
    return hipErrorInvalidValue;
}

}  // namespace idf
