// Measurement aids: kernels of known work that show what the machine sustains, so that a benchmark can report its
// kernels against a measured ceiling next to the data-sheet one.  Not part of the training step.
#include "common.h"

namespace rn50 {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kProbeAcc = 4;      // independent accumulators per wavefront: no MFMA waits for the one before it
constexpr int kProbeUnroll = 8;

// Nothing but matrix instructions: every wavefront issues iters * kProbeUnroll * kProbeAcc MFMAs on register operands.
template <bool BF>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *__restrict__ sink, int iters, float a, float b, long long *__restrict__ ticks)
{
    floatx16 acc[kProbeAcc];
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    const float x = a + threadIdx.x * 1e-9f, y = b;
    bf16x8 xb, yb;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        xb[e] = (__bf16)x;
        yb[e] = (__bf16)y;
    }
    // shader-clock cycles and ticks of the constant 100 MHz reference counter around the loop: their ratio is the clock the
    // loop ran at
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u)
#pragma unroll
            for (int i = 0; i < kProbeAcc; ++i) {
                if (BF) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xb, yb, acc[i], 0, 0, 0);
                else acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[i], 0, 0, 0);
            }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kProbeAcc; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    const long long c1 = clock64(), w1 = wall_clock64();  // after the accumulators are read: the last MFMA has finished
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (ticks && blockIdx.x == 0 && threadIdx.x == 0) {
        ticks[0] = c1 - c0;
        ticks[1] = w1 - w0;
    }
}

// dst[i] = src[i], one 16-byte element per lane and no loop: count4 float4 elements read once and written once.  (Of the
// forms measured on the MI355X this plain one is the fastest: 6.1-6.2 TB/s at 1 GiB against 4.7-4.8 for a grid-stride loop
// over 16384 workgroups, 3.6 for eight loads in flight per lane and 5.1 for the runtime's own device-to-device copy.)
__global__ __launch_bounds__(256) void probe_copy_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t count4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count4) dst[i] = src[i];
}

// A kernel that does nothing: launched back to back on one stream it shows what a dependent launch costs at least.
__global__ void probe_empty_kernel(float *sink)
{
    if (sink && threadIdx.x == 9999u) sink[0] = 1.f;  // never true: keeps the argument alive
}

}  // namespace rn50

using namespace rn50;

extern "C" int rn50_probe_empty(int workgroups, int launches, float *sink, void *stream)
{
    RN50_REQUIRE(workgroups > 0 && workgroups <= (1 << 20), RN50_EINVAL, "rn50_probe_empty: workgroups must be in [1, 2^20]");
    RN50_REQUIRE(launches > 0 && launches <= (1 << 16), RN50_EINVAL, "rn50_probe_empty: launches must be in [1, 2^16]");
    for (int i = 0; i < launches; ++i) hipLaunchKernelGGL(probe_empty_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, sink);
    return launch_status("rn50_probe_empty");
}

extern "C" int rn50_probe_mfma(int dtype, int iters, int wgs_per_cu, float *sink, long long *ticks_or_null, double *flop_out, void *stream)
{
    RN50_REQUIRE(dtype == RN50_DTYPE_F32 || dtype == RN50_DTYPE_BF16, RN50_EINVAL, "rn50_probe_mfma: unknown dtype");
    RN50_REQUIRE(iters > 0 && iters <= (1 << 24) && wgs_per_cu > 0 && wgs_per_cu <= 8, RN50_EINVAL,
                 "rn50_probe_mfma: iters must be in [1, 2^24] and wgs_per_cu in [1, 8]");
    RN50_REQUIRE(sink && aligned16(sink), RN50_EINVAL, "rn50_probe_mfma: sink must be non-null and 16-byte aligned");
    RN50_REQUIRE(((uintptr_t)ticks_or_null & 7) == 0, RN50_EINVAL, "rn50_probe_mfma: ticks must be 8-byte aligned");
    const int grid = 256 * wgs_per_cu;
    const double k_per_mfma = dtype == RN50_DTYPE_BF16 ? 16.0 : 2.0;
    if (flop_out) *flop_out = (double)grid * 4.0 * iters * kProbeUnroll * kProbeAcc * (32.0 * 32.0 * k_per_mfma * 2.0);
    if (dtype == RN50_DTYPE_BF16) hipLaunchKernelGGL((probe_mfma_kernel<true>), dim3(grid), dim3(256), 0, (hipStream_t)stream, sink, iters, 1.f, 1.f, ticks_or_null);
    else hipLaunchKernelGGL((probe_mfma_kernel<false>), dim3(grid), dim3(256), 0, (hipStream_t)stream, sink, iters, 1.f, 1.f, ticks_or_null);
    return launch_status("rn50_probe_mfma");
}

extern "C" int rn50_probe_copy(size_t count, const float *src, float *dst, void *stream)
{
    RN50_REQUIRE(src && dst && aligned16(src) && aligned16(dst), RN50_EINVAL, "rn50_probe_copy: pointers must be non-null and 16-byte aligned");
    RN50_REQUIRE(count > 0 && count % 4 == 0, RN50_EINVAL, "rn50_probe_copy: count must be a positive multiple of 4");
    RN50_REQUIRE(count <= ((size_t)1 << 40), RN50_EUNSUPPORTED, "rn50_probe_copy: count too large");
    const size_t count4 = count / 4;
    const unsigned grid = (unsigned)((count4 + 255) / 256);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const float4 *)src, (float4 *)dst, count4);
    return launch_status("rn50_probe_copy");
}
