// Measurement aid: what rate of dense 16-bit MFMA work does this GPU sustain?  The published peak assumes the
// maximum clock; under a chip-wide matrix-core load the clock settles lower.  The probe runs the instruction
// the second-moment kernel is made of (v_mfma_f32_16x16x32_f16, independent accumulators, two waves per
// SIMD on every compute unit) and nothing else, so its rate is the ceiling that kernel can approach.
#include "llla_common.hpp"
#include "llla_measure.h"

namespace llla {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeWorkgroups = 4096;     // 16 per compute unit, two resident at a time
constexpr int kProbeMfmaPerIter = 8;

__global__ __launch_bounds__(256, 2) void mfma_rate_kernel(int iters, float *__restrict__ sink)
{
    const int tid = threadIdx.x;
    half8 a, b;
#pragma unroll
    for (int t = 0; t < 8; ++t) { a[t] = (_Float16)(0.001f * ((tid + t) & 15)); b[t] = (_Float16)(0.002f * ((tid + 3 * t) & 7)); }
    f32x4 acc[kProbeMfmaPerIter];
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kProbeMfmaPerIter; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[m], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m) s += acc[m][0] + acc[m][1] + acc[m][2] + acc[m][3];
    if (s == 12345.678f) sink[0] = s;       // keeps the accumulators alive; never true for these operands
}

// Plain copy of known size: what the HBM counters (FETCH_SIZE, WRITE_SIZE) read per byte moved.
__global__ __launch_bounds__(256) void copy_rate_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace llla

extern "C" llla_status llla_probe_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst) return LLLA_ERR_NULL;
    if (bytes == 0 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return LLLA_ERR_PARAM;
    using namespace llla;
    copy_rate_kernel<<<4096, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? LLLA_OK : LLLA_ERR_LAUNCH;
}

extern "C" llla_status llla_probe_mfma_f16(int iters, void *scratch, double *flops, void *stream)
{
    if (!scratch || !flops) return LLLA_ERR_NULL;
    if (iters <= 0 || iters > (1 << 20)) return LLLA_ERR_PARAM;
    using namespace llla;
    mfma_rate_kernel<<<kProbeWorkgroups, 256, 0, static_cast<hipStream_t>(stream)>>>(iters, static_cast<float *>(scratch));
    *flops = (double)kProbeWorkgroups * 4.0 * iters * kProbeMfmaPerIter * (2.0 * 16 * 16 * 32);
    return hipGetLastError() == hipSuccess ? LLLA_OK : LLLA_ERR_LAUNCH;
}
