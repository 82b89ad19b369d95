// Matrix-core event propagation for one arriving row of a 3x3, stride 1, same-padded conv layer
// (bfloat16 events and weights -> float32 state, or int8 -> int32).
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
//   * The retained rows of c (rows y-1 and y of the rolling buffer) are fetched at the start and
//     are in flight during the contraction.  Epilogue: the row that is now final (y-1; also y
//     when y is the last row of the sample) is activated, rounded to the event type and emitted
//     -- through a fused 2x2 max-pool when one follows -- and forgotten; the others go back to
//     the rolling buffer; row y+1 is started from the bias.
#include "idf.h"
#include "idf_kernels.h"

namespace idf {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

struct TraitsBf16 {
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
    {
        int n = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) { n += (v[i] & 0x7fff) != 0; n += (v[i] & 0x7fff0000) != 0; }
        return n;
    }
    static __device__ __forceinline__ st_t activate(st_t c, int act, int, int) { return act == IDF_ACT_NONE ? c : fmaxf(c, 0.f); }
    static __device__ __forceinline__ ev_t to_ev(st_t h)
    {
        uint32_t u = __float_as_uint(h);
        u += 0x7fffu + ((u >> 16) & 1u);           // round to nearest, ties to even
        return (ev_t)(u >> 16);
    }
    static __device__ __forceinline__ st_t ev_val(ev_t v) { return __uint_as_float((uint32_t)v << 16); }
    static __device__ __forceinline__ bool ev_nonzero(ev_t v) { return (v & 0x7fffu) != 0; }
};

struct TraitsI8 {
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
        int n = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int b = 0; b < 4; ++b) n += ((v[i] >> (8 * b)) & 0xff) != 0;
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
};

constexpr int kMaxPos = 128 + 2;                 // positions of the widest tile plus halo
constexpr int kNzWords = (kMaxPos + 31) / 32 + 1;

template <class T, int WM, int WN>
__global__ void __launch_bounds__(64 * WM * WN) k_conv3x3_mfma(const MfmaStep a, const StreamSel sel)
{
    using acc_t = typename T::acc_t; using st_t = typename T::st_t; using ev_t = typename T::ev_t;
    constexpr int VL = T::VL, EB = T::EB, KI = 2 * VL;
    constexpr int MT = 32 * WM, NC = 32 * WN, NT = 64 * WM * WN;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ uint32_t nz[64][kNzWords];          // per channel chunk: positions with a non-zero cell
    __shared__ unsigned long long red[2][WM * WN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int si = blockIdx.z;
    const int stream = sel_stream(sel, si);
    const int n_co_chunks = (a.c_out + NC - 1) / NC;
    const int x_tile = blockIdx.x / n_co_chunks, co_chunk = blockIdx.x - x_tile * n_co_chunks;
    const int x0 = x_tile * MT, co0 = co_chunk * NC;
    const int W = a.w, C_in = a.c_in, C_out = a.c_out;
    const int chunks = C_in / VL;                  // 16-byte cells per position
    const int xs_stride = C_in * EB + 16;          // bytes per position in LDS (padded against bank conflicts)

    // ---- retained rows: issue the loads now, use them in the epilogue ---------------------
    const int row_lane = (lane >> 5) * 4;          // D layout: row = 8*i + (lane/32)*4 + j, col = lane%32
    const int xo_base = x0 + wm * 32 + row_lane;
    const int co = co0 + wn * 32 + (lane & 31);
    const bool co_ok = co < C_out;
    st_t *ring = (st_t *)a.ring + (int64_t)stream * a.ring_stream_stride;
    st_t init[3][16];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
        const bool rd = a.t[ky].valid && !a.t[ky].fresh;
        const st_t b0 = a.bias && co_ok ? ((const st_t *)a.bias)[co] : (st_t)0;
        const st_t *rrow = ring + (int64_t)a.t[ky].ring_slot * W * C_out;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int xo = xo_base + 8 * i + j;
                init[ky][i * 4 + j] = (rd && co_ok && xo < W) ? rrow[(int64_t)xo * C_out + co] : b0;
            }
    }

    // ---- input row stretch [x0-1, x0+MT+1) -> LDS, with occupancy bits ----------------------
    const int64_t in_idx = a.in_by_position ? (int64_t)(sel.pos0 + si) : (int64_t)stream;
    const unsigned char *in_row = (const unsigned char *)a.in + (in_idx * a.in_stream_stride + a.in_row_off) * EB;
    for (int i = tid; i < chunks * kNzWords; i += NT) nz[i / kNzWords][i % kNzWords] = 0;
    __syncthreads();
    const bool small_c = C_in < VL;                // first layers: 1..4 input channels
    {
        const bool count = co_chunk == 0 && a.stats;
        unsigned long long ev = 0, taps = 0;
        if (!small_c) {
            const int cells = (MT + 2) * chunks;
            for (int i = tid; i < cells; i += NT) {
                const int p = i / chunks, c = i - p * chunks;
                const int x = x0 - 1 + p;
                i32x4 v = {0, 0, 0, 0};
                if (x >= 0 && x < W) v = *reinterpret_cast<const i32x4 *>(in_row + ((int64_t)x * C_in + c * VL) * EB);
                *reinterpret_cast<i32x4 *>(smem + p * xs_stride + c * 16) = v;
                if (T::cell_nonzero(v)) {
                    atomicOr(&nz[c][p >> 5], 1u << (p & 31));
                    if (count && p >= 1 && p <= MT) {
                        const int n = T::count_nonzero(v);
                        ev += n;
                        taps += n * (3 - (x == 0) - (x == W - 1));
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
                if (x >= 0 && x < W) v = in_e[(int64_t)x * C_in + (i - p * C_in)];
                xs_e[i] = v;
                if (count && p >= 1 && p <= MT && T::ev_nonzero(v)) {
                    ev += 1;
                    taps += 3 - (x == 0) - (x == W - 1);
                }
            }
        }
        if (count) {
            for (int off = 32; off > 0; off >>= 1) { ev += __shfl_down(ev, off); taps += __shfl_down(taps, off); }
            if (lane == 0) { red[0][wave] = ev; red[1][wave] = taps; }
        }
        __syncthreads();
        if (count && tid == 0) {
            unsigned long long e = 0, t = 0;
            for (int wv = 0; wv < WM * WN; ++wv) { e += red[0][wv]; t += red[1][wv]; }
            unsigned long long *dst = a.stats + ((int64_t)stream * a.n_layers + a.layer) * 2;
            if (e) atomicAdd(dst, e);
            if (t) atomicAdd(dst + 1, t * (unsigned long long)(a.taps_y * C_out));
        }
    }

    // ---- which K-steps have anything in them for this wave's 32 positions -------------------
    const int KT = 3 * C_in;
    const int steps = (KT + KI - 1) / KI;
    unsigned long long live;
    {
        bool occ = small_c && lane < steps;          // few channels: every step is visited
        if (!small_c && lane < steps) {
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
                const int k0 = lane * KI + hlf * VL;
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
    }

    // ---- contraction over the live K-steps ----------------------------------------------------
    acc_t acc[3];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[ky][q] = 0;
    const int hlf = lane >> 5, r = wm * 32 + (lane & 31);
    const unsigned char *wbase = (const unsigned char *)a.wfrag + ((int64_t)hlf * a.c_out_pad + co0 + wn * 32 + (lane & 31)) * 16;
    const int64_t w_step = (int64_t)2 * a.c_out_pad * 16;           // bytes per K-step
    const int64_t w_ky = (int64_t)steps * w_step;                    // bytes per ky
    // Operands of the next live steps are fetched kDepth steps ahead of their use.
    constexpr int kDepth = 4;
    int sq[kDepth];
    i32x4 aq[kDepth], bq[kDepth][3];
    auto fetch = [&](int d) {
        if (live) {
            const int s = __builtin_ctzll(live);
            live &= live - 1;
            sq[d] = s;
            const int k0 = s * KI + hlf * VL;
            const int kx = k0 / C_in, ci = k0 - kx * C_in;
            aq[d] = i32x4{0, 0, 0, 0};
            if (small_c) {
                const ev_t *xs_e = reinterpret_cast<const ev_t *>(smem) + r * C_in;
                ev_t e[VL];
#pragma unroll
                for (int q = 0; q < VL; ++q) e[q] = k0 + q < KT ? xs_e[k0 + q] : (ev_t)0;
                __builtin_memcpy(&aq[d], e, 16);
            } else if (k0 < KT) {
                aq[d] = *reinterpret_cast<const i32x4 *>(smem + (r + kx) * xs_stride + ci * EB);
            }
            const unsigned char *wp = wbase + s * w_step;
            bq[d][0] = *reinterpret_cast<const i32x4 *>(wp);
            bq[d][1] = *reinterpret_cast<const i32x4 *>(wp + w_ky);
            bq[d][2] = *reinterpret_cast<const i32x4 *>(wp + 2 * w_ky);
        } else {
            sq[d] = -1;
        }
    };
#pragma unroll
    for (int d = 0; d < kDepth; ++d) fetch(d);
    for (bool more = true; more;) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            if (sq[d] < 0) { more = false; break; }
            acc[0] = T::mfma(aq[d], bq[d][0], acc[0]);
            acc[1] = T::mfma(aq[d], bq[d][1], acc[1]);
            acc[2] = T::mfma(aq[d], bq[d][2], acc[2]);
            fetch(d);
        }
    }

    // ---- epilogue -----------------------------------------------------------------------------
    ev_t *held = (ev_t *)a.held + (int64_t)stream * a.held_stream_stride;
    ev_t hprev[16];                                   // activations of the even row finalised by tap 2
#pragma unroll
    for (int q = 0; q < 16; ++q) hprev[q] = 0;
#pragma unroll
    for (int kk = 0; kk < 3; ++kk) {
        const int ky = 2 - kk;                        // row y-1 first
        const MfmaTap &t = a.t[ky];
        if (!t.valid) continue;
        st_t c[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) c[q] = init[ky][q] + acc[ky][q];
        if (t.emit == kEmitNone) {
            st_t *rrow = ring + (int64_t)t.ring_slot * W * C_out;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int xo = xo_base + 8 * i + j;
                    if (co_ok && xo < W) rrow[(int64_t)xo * C_out + co] = c[i * 4 + j];
                }
            continue;
        }
        st_t h[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) h[q] = T::activate(c[q], a.act, a.shr, a.clamp_hi);
        if (a.pool_layer >= 0 && a.stats) {          // what the fused pool receives counts as its events
            unsigned int n = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    n += (co_ok && xo_base + 8 * i + j < W && T::ev_nonzero(T::to_ev(h[i * 4 + j]))) ? 1u : 0u;
            for (int off = 32; off > 0; off >>= 1) n += __shfl_down(n, off);
            if (lane == 0 && n)
                atomicAdd(a.stats + ((int64_t)stream * a.n_layers + a.pool_layer) * 2, (unsigned long long)n);
        }
        if (t.emit == kEmitDirect) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int xo = xo_base + 8 * i + j;
                    if (!(co_ok && xo < W)) continue;
                    const int64_t off = (int64_t)stream * a.dst_stream_stride + (t.dst_slot * W + xo) * C_out + co;
                    if (a.to_output) ((st_t *)a.dst)[off] = h[i * 4 + j];
                    else ((ev_t *)a.dst)[off] = T::to_ev(h[i * 4 + j]);
                }
        } else if (t.emit == kEmitHold) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int xo = xo_base + 8 * i + j;
                    const ev_t e = T::to_ev(h[i * 4 + j]);
                    hprev[i * 4 + j] = e;
                    if (t.store_held && co_ok && xo < W) held[(int64_t)xo * C_out + co] = e;
                }
        } else {   // pool with the held row (kEmitPoolHeld) or with the row finalised a moment ago (kEmitPoolReg)
            const int Wp = W / 2;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 2; ++jj) {
                    const int xo = xo_base + 8 * i + 2 * jj;
                    const int xp = xo >> 1;
                    if (!(co_ok && xp < Wp)) continue;
                    st_t m = T::ev_val(T::to_ev(h[i * 4 + 2 * jj]));
                    const st_t m1 = T::ev_val(T::to_ev(h[i * 4 + 2 * jj + 1]));
                    m = m1 > m ? m1 : m;
                    st_t e0, e1;
                    if (t.emit == kEmitPoolHeld) {
                        e0 = T::ev_val(held[(int64_t)xo * C_out + co]);
                        e1 = T::ev_val(held[(int64_t)(xo + 1) * C_out + co]);
                    } else {
                        e0 = T::ev_val(hprev[i * 4 + 2 * jj]);
                        e1 = T::ev_val(hprev[i * 4 + 2 * jj + 1]);
                    }
                    m = e0 > m ? e0 : m;
                    m = e1 > m ? e1 : m;
                    const int64_t off = (int64_t)stream * a.dst_stream_stride + (t.dst_slot * Wp + xp) * C_out + co;
                    if (a.to_output) ((st_t *)a.dst)[off] = m;
                    else ((ev_t *)a.dst)[off] = T::to_ev(m);
                }
        }
    }
}

template <class T, int WM, int WN>
hipError_t launch_one(const MfmaStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    constexpr int MT = 32 * WM, NC = 32 * WN;
    const int x_tiles = (a.w + MT - 1) / MT, co_chunks = (a.c_out + NC - 1) / NC;
    const size_t lds = (size_t)(MT + 2) * (a.c_in * T::EB + 16);
    return launch(k_conv3x3_mfma<T, WM, WN>, dim3(x_tiles * co_chunks, 1, sel.n), dim3(64 * WM * WN), lds, lc, a, sel);
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

bool conv3x3_mfma_eligible(int prec, const Geom &g)
{
    if (prec != IDF_PREC_BF16 && prec != IDF_PREC_I8) return false;
    const int vl = prec == IDF_PREC_BF16 ? 8 : 16;
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

// Weights [k_h][k_w][c_in][c_out] -> fragment order [ky][k/VL][c_out_pad][VL] with k = kx*c_in + ci,
// zero padded to whole K-steps and to a multiple of 64 output channels.
size_t conv3x3_mfma_pack(int prec, const Geom &g, const void *w_khkwcico, void *out)
{
    const int vl = prec == IDF_PREC_BF16 ? 8 : 16, eb = prec == IDF_PREC_BF16 ? 2 : 1;
    const int KT = 3 * g.c_in, steps = (KT + 2 * vl - 1) / (2 * vl), kc = 2 * steps;
    const int cop = (g.c_out + 63) / 64 * 64;
    const size_t bytes = (size_t)3 * kc * cop * 16;
    if (!out) return bytes;
    unsigned char *o = (unsigned char *)out;
    const unsigned char *src = (const unsigned char *)w_khkwcico;
    for (size_t i = 0; i < bytes; ++i) o[i] = 0;
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

hipError_t launch_conv3x3_mfma(int prec, const MfmaStep &a, const StreamSel &sel, const LaunchCtx &lc)
{
    if (prec == IDF_PREC_BF16) return launch_prec<TraitsBf16>(a, sel, lc);
    if (prec == IDF_PREC_I8) return launch_prec<TraitsI8>(a, sel, lc);
    return hipErrorInvalidValue;
}

}  // namespace idf
