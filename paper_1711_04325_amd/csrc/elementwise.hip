// Bandwidth-bound flat-arena kernels: half-precision communication buffer (Section 3, "Software")
// and the update rule of Appendix A.1.  One launch covers the whole 25.6 M-element arena.
#include "common.h"

namespace rn50 {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 256 * 16;  // 256 CUs, enough resident waves per CU to cover HBM latency

union H8 { uint4 v; _Float16 h[8]; uint16_t u[8]; };

// 8 elements per thread per iteration: two 16-byte loads, one 16-byte store.
__global__ __launch_bounds__(kThreads) void pack_fp16_kernel(size_t count, const float *__restrict__ g,
                                                              uint16_t *__restrict__ out)
{
    const size_t n8 = count / 8;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += stride) {
        const float4 a = reinterpret_cast<const float4 *>(g)[2 * i];
        const float4 b = reinterpret_cast<const float4 *>(g)[2 * i + 1];
        H8 o;
        o.h[0] = (_Float16)a.x; o.h[1] = (_Float16)a.y; o.h[2] = (_Float16)a.z; o.h[3] = (_Float16)a.w;
        o.h[4] = (_Float16)b.x; o.h[5] = (_Float16)b.y; o.h[6] = (_Float16)b.z; o.h[7] = (_Float16)b.w;
        reinterpret_cast<uint4 *>(out)[i] = o.v;
    }
    if (blockIdx.x == 0) {  // ragged tail (< 8 elements)
        const size_t i = n8 * 8 + threadIdx.x;
        if (i < count) {
            union { _Float16 h; uint16_t u; } c;
            c.h = (_Float16)g[i];
            out[i] = c.u;
        }
    }
}

__global__ __launch_bounds__(kThreads) void unpack_fp16_kernel(size_t count, const uint16_t *__restrict__ in,
                                                                float scale, float *__restrict__ g)
{
    const size_t n8 = count / 8;
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n8; i += stride) {
        H8 v;
        v.v = reinterpret_cast<const uint4 *>(in)[i];
        float4 a, b;
        a.x = (float)v.h[0] * scale; a.y = (float)v.h[1] * scale; a.z = (float)v.h[2] * scale; a.w = (float)v.h[3] * scale;
        b.x = (float)v.h[4] * scale; b.y = (float)v.h[5] * scale; b.z = (float)v.h[6] * scale; b.w = (float)v.h[7] * scale;
        reinterpret_cast<float4 *>(g)[2 * i] = a;
        reinterpret_cast<float4 *>(g)[2 * i + 1] = b;
    }
    if (blockIdx.x == 0) {
        const size_t i = n8 * 8 + threadIdx.x;
        if (i < count) {
            union { _Float16 h; uint16_t u; } c;
            c.u = in[i];
            g[i] = (float)c.h * scale;
        }
    }
}

struct OptP { float eta, mu1, mu2, one_minus_mu2, eps, a_sgd, a_rms, wd, g_scale; };

__device__ inline void update_one(const OptP &p, float gi, bool decay, float &th, float &de, float &mm)
{
    gi *= p.g_scale;
    if (decay) gi = fmaf(p.wd, th, gi);
    mm = fmaf(p.mu2, mm, p.one_minus_mu2 * gi * gi);
    const float coef = p.a_sgd + p.a_rms / (sqrtf(mm) + p.eps);
    de = fmaf(p.mu1, de, -coef * gi);
    th = fmaf(p.eta, de, th);
}

// 4 elements per thread per iteration.  HALF selects the fused unpack of the half-precision buffer.
template <bool HALF>
__global__ __launch_bounds__(kThreads) void opt_update_kernel(size_t count, float *__restrict__ theta,
                                                              float *__restrict__ delta, float *__restrict__ m,
                                                              const float *__restrict__ g, const uint16_t *__restrict__ g16,
                                                              const uint8_t *__restrict__ wd_mask, OptP p)
{
    const size_t n4 = count / 4;
    const size_t stride = (size_t)gridDim.x * kThreads;
    const bool any_decay = p.wd != 0.0f;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += stride) {
        float4 th = reinterpret_cast<float4 *>(theta)[i];
        float4 de = reinterpret_cast<float4 *>(delta)[i];
        float4 mm = reinterpret_cast<float4 *>(m)[i];
        float4 gi;
        if (HALF) {
            union { uint2 v; _Float16 h[4]; } u;
            u.v = reinterpret_cast<const uint2 *>(g16)[i];
            gi = make_float4((float)u.h[0], (float)u.h[1], (float)u.h[2], (float)u.h[3]);
        } else {
            gi = reinterpret_cast<const float4 *>(g)[i];
        }
        const bool decay = any_decay && (wd_mask == nullptr || wd_mask[(i * 4) / RN50_WD_GROUP] != 0);
        update_one(p, gi.x, decay, th.x, de.x, mm.x);
        update_one(p, gi.y, decay, th.y, de.y, mm.y);
        update_one(p, gi.z, decay, th.z, de.z, mm.z);
        update_one(p, gi.w, decay, th.w, de.w, mm.w);
        reinterpret_cast<float4 *>(theta)[i] = th;
        reinterpret_cast<float4 *>(delta)[i] = de;
        reinterpret_cast<float4 *>(m)[i] = mm;
    }
    if (blockIdx.x == 0) {
        const size_t i = n4 * 4 + threadIdx.x;
        if (i < count) {
            float gi;
            if (HALF) {
                union { _Float16 h; uint16_t u; } c;
                c.u = g16[i];
                gi = (float)c.h;
            } else {
                gi = g[i];
            }
            const bool decay = any_decay && (wd_mask == nullptr || wd_mask[i / RN50_WD_GROUP] != 0);
            update_one(p, gi, decay, theta[i], delta[i], m[i]);
        }
    }
}

static int flat_grid(size_t count, int per_thread)
{
    size_t blocks = (count / per_thread + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > (size_t)kMaxBlocks) blocks = kMaxBlocks;
    return (int)blocks;
}

}  // namespace rn50

using namespace rn50;

extern "C" int grad_pack_fp16(size_t count, const float *g, uint16_t *out16, void *stream)
{
    if (count == 0) return RN50_OK;
    RN50_REQUIRE(g && out16, RN50_EINVAL, "grad_pack_fp16: null pointer");
    RN50_REQUIRE(aligned16(g) && aligned16(out16), RN50_EINVAL, "grad_pack_fp16: pointers must be 16-byte aligned");
    hipLaunchKernelGGL(pack_fp16_kernel, dim3(flat_grid(count, 8)), dim3(kThreads), 0, (hipStream_t)stream, count, g, out16);
    return launch_status("grad_pack_fp16");
}

extern "C" int grad_unpack_fp16(size_t count, const uint16_t *in16, float scale, float *g, void *stream)
{
    if (count == 0) return RN50_OK;
    RN50_REQUIRE(g && in16, RN50_EINVAL, "grad_unpack_fp16: null pointer");
    RN50_REQUIRE(aligned16(g) && aligned16(in16), RN50_EINVAL, "grad_unpack_fp16: pointers must be 16-byte aligned");
    hipLaunchKernelGGL(unpack_fp16_kernel, dim3(flat_grid(count, 8)), dim3(kThreads), 0, (hipStream_t)stream, count, in16, scale, g);
    return launch_status("grad_unpack_fp16");
}

extern "C" int opt_update(size_t count, float *theta, float *delta, float *m, const float *g_or_null,
                          const uint16_t *g16_or_null, const uint8_t *wd_mask_or_null, const rn50_opt_hparams *hp,
                          void *stream)
{
    RN50_REQUIRE(hp, RN50_EINVAL, "opt_update: null hyper-parameters");
    RN50_REQUIRE((g_or_null != nullptr) != (g16_or_null != nullptr), RN50_EINVAL,
                 "opt_update: exactly one of g and g16 must be given");
    if (count == 0) return RN50_OK;
    RN50_REQUIRE(theta && delta && m, RN50_EINVAL, "opt_update: null state pointer");
    RN50_REQUIRE(aligned16(theta) && aligned16(delta) && aligned16(m) && aligned16(g_or_null) && aligned16(g16_or_null),
                 RN50_EINVAL, "opt_update: pointers must be 16-byte aligned");
    OptP p{hp->eta, hp->mu1, hp->mu2, 1.0f - hp->mu2, hp->eps, hp->a_sgd, hp->a_rms, hp->wd, hp->g_scale};
    const dim3 grid(flat_grid(count, 4)), block(kThreads);
    if (g16_or_null)
        hipLaunchKernelGGL(opt_update_kernel<true>, grid, block, 0, (hipStream_t)stream, count, theta, delta, m,
                           (const float *)nullptr, g16_or_null, wd_mask_or_null, p);
    else
        hipLaunchKernelGGL(opt_update_kernel<false>, grid, block, 0, (hipStream_t)stream, count, theta, delta, m,
                           g_or_null, (const uint16_t *)nullptr, wd_mask_or_null, p);
    return launch_status("opt_update");
}
