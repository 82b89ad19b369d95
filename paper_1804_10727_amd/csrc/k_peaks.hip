// Plain kernels that show what this machine delivers to code with nothing else to do: a 16-byte
// copy, chains of float32 multiply-adds on the vector units, and chains of the three matrix
// instructions the conv kernel uses.  Their rates are quoted next to the published peaks the
// rooflines are priced against; nothing on the hot path calls them.
#include "idf.h"
#include "idf_kernels.h"

namespace idf {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(16))) int i32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kPeakThreads = 256;        // four waves, one per SIMD
constexpr int kPeakChains = 4;           // independent accumulator sets per wave: an instruction never waits for its own result

// Every lane keeps kPeakChains accumulator tiles going; what they hold at the end is written out
// (one value per lane) so that the loop cannot be dropped.
template <int KIND>
__global__ void __launch_bounds__(kPeakThreads) k_peak_mfma(float *sink, int iters)
{
    const int lane = threadIdx.x;
    const i32x4 a = {lane + 1, lane + 2, lane + 3, lane + 4};          // any bit patterns: the rate does not depend on the values
    const i32x4 b = {lane + 5, lane + 6, lane + 7, lane + 8};
    if constexpr (KIND == IDF_PEAK_MFMA_I8) {
        i32x16 acc[kPeakChains];
#pragma unroll
        for (int c = 0; c < kPeakChains; ++c)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[c][q] = c;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int c = 0; c < kPeakChains; ++c) acc[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[c], 0, 0, 0);
        int s = 0;
#pragma unroll
        for (int c = 0; c < kPeakChains; ++c)
#pragma unroll
            for (int q = 0; q < 16; ++q) s += acc[c][q];
        sink[blockIdx.x * kPeakThreads + threadIdx.x] = (float)s;
    } else {
        f32x16 acc[kPeakChains];
#pragma unroll
        for (int c = 0; c < kPeakChains; ++c)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[c][q] = (float)c;
        // bfloat16 operands: small normal numbers (exponent field 0x3c..0x3f), so nothing overflows on the way
        const i32x4 ah = {0x3c003c80, 0x3d003d80, 0x3c803c00, 0x3d803d00}, bh = {0x3d003c00, 0x3c803d80, 0x3d803c80, 0x3c003d00};
        const float af = 1.0f / (float)(lane + 2), bf = 1.0f / (float)(lane + 3);
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int c = 0; c < kPeakChains; ++c) {
                if constexpr (KIND == IDF_PEAK_MFMA_BF16)
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ah), __builtin_bit_cast(bf16x8, bh), acc[c], 0, 0, 0);
                else
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(af, bf, acc[c], 0, 0, 0);
            }
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < kPeakChains; ++c)
#pragma unroll
            for (int q = 0; q < 16; ++q) s += acc[c][q];
        sink[blockIdx.x * kPeakThreads + threadIdx.x] = s;
    }
}

constexpr int kFmaChains = 16;           // independent multiply-add chains per lane
__global__ void __launch_bounds__(kPeakThreads) k_peak_fma(float *sink, int iters)
{
    float v[kFmaChains];
    const float m = 1.0f - 1.0f / (float)(threadIdx.x + 1024), add = 1.0f / (float)(threadIdx.x + 7);
#pragma unroll
    for (int c = 0; c < kFmaChains; ++c) v[c] = (float)c;
    for (int it = 0; it < iters; ++it)
#pragma unroll
        for (int c = 0; c < kFmaChains; ++c) v[c] = __builtin_fmaf(v[c], m, add);
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kFmaChains; ++c) s += v[c];
    sink[blockIdx.x * kPeakThreads + threadIdx.x] = s;
}

// dst[i] = src[i] in 16-byte pieces, grid-stride.  (Four pieces per lane in flight with
// non-temporal accesses measured slower: 4.5 against 5.0 TB/s on 2 GiB.)
__global__ void __launch_bounds__(kPeakThreads) k_peak_copy(const i32x4 *src, i32x4 *dst, size_t n16)
{
    const size_t step = (size_t)gridDim.x * kPeakThreads;
    for (size_t i = (size_t)blockIdx.x * kPeakThreads + threadIdx.x; i < n16; i += step) dst[i] = src[i];
}

}  // namespace

size_t peak_sink_bytes(int blocks) { return (size_t)blocks * kPeakThreads * sizeof(float); }

// Operations (multiply and add counted separately) one launch of `blocks` workgroups performs.
double peak_ops(int kind, int blocks, int iters)
{
    const double waves = (double)blocks * (kPeakThreads / 64);
    switch (kind) {
    case IDF_PEAK_FMA_F32: return 2.0 * (double)blocks * kPeakThreads * kFmaChains * iters;
    case IDF_PEAK_MFMA_F32: return 2.0 * 32 * 32 * 2 * kPeakChains * waves * iters;
    case IDF_PEAK_MFMA_BF16: return 2.0 * 32 * 32 * 16 * kPeakChains * waves * iters;
    case IDF_PEAK_MFMA_I8: return 2.0 * 32 * 32 * 32 * kPeakChains * waves * iters;
    default: return 0.0;
    }
}

hipError_t launch_peak(int kind, void *buf, size_t bytes, int blocks, int iters, const LaunchCtx &lc)
{
    const dim3 grid(blocks), block(kPeakThreads);
    switch (kind) {
    case IDF_PEAK_COPY: {
        const size_t n16 = bytes / 32;                               // first half -> second half
        return launch(k_peak_copy, grid, block, 0, lc, (const i32x4 *)buf, (i32x4 *)buf + n16, n16);
    }
    case IDF_PEAK_FMA_F32: return launch(k_peak_fma, grid, block, 0, lc, (float *)buf, iters);
    case IDF_PEAK_MFMA_F32: return launch(k_peak_mfma<IDF_PEAK_MFMA_F32>, grid, block, 0, lc, (float *)buf, iters);
    case IDF_PEAK_MFMA_BF16: return launch(k_peak_mfma<IDF_PEAK_MFMA_BF16>, grid, block, 0, lc, (float *)buf, iters);
    case IDF_PEAK_MFMA_I8: return launch(k_peak_mfma<IDF_PEAK_MFMA_I8>, grid, block, 0, lc, (float *)buf, iters);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace idf
