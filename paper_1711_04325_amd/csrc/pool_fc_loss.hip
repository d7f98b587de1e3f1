// The layers of ResNet-50 (He et al. 2016) around the convolutions: 3x3/2 max pooling, global average
// pooling, the 1000-way fully connected layer and the softmax cross-entropy loss.  NHWC, fp32.
#include "common.h"

namespace rn50 {

// one thread per (n, p, q, 4 channels).  INAFF: the pooled tensor is max(0, x*in_scale[c] + in_shift[c]), the BN + ReLU
// in front of the pooling layer applied to every value as it is loaded.
template <class T, bool INAFF>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(int N, int C4, int H, int W, int P, int Q, const T *__restrict__ x,
                                                          const float *__restrict__ in_scale, const float *__restrict__ in_shift,
                                                          T *__restrict__ y, uint8_t *__restrict__ arg)
{
    // overlapping windows re-read their neighbours' pixels: keep neighbours on one XCD
    const size_t i = (size_t)xcd_contiguous(blockIdx.x, gridDim.x) * 256 + threadIdx.x;
    if (i >= (size_t)N * P * Q * C4) return;
    // 32-bit index arithmetic (the host checks the element count): 64-bit divisions cost more than the nine loads
    const unsigned iu = (unsigned)i;
    const int c = (int)(iu % (unsigned)C4);
    unsigned t = iu / (unsigned)C4;
    const int q = (int)(t % (unsigned)Q);
    t /= (unsigned)Q;
    const int p = (int)(t % (unsigned)P), n = (int)(t / (unsigned)P);
    float best[4] = {0.f, 0.f, 0.f, 0.f};
    int bi[4] = {-1, -1, -1, -1};
    float4 sc = make_float4(0.f, 0.f, 0.f, 0.f), sh = sc;
    if (INAFF) {
        sc = ld4(in_scale, c);
        sh = ld4(in_shift, c);
    }
    // all nine loads first (a tap outside the image loads a clamped pixel and is skipped below), so that they are in
    // flight together
    float4 tap[9];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int h = min(max(2 * p + r - 1, 0), H - 1), w = min(max(2 * q + s - 1, 0), W - 1);
            tap[r * 3 + s] = ld4(x, ((size_t)(n * H + h) * W + w) * C4 + c);
        }
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int h = 2 * p + r - 1, w = 2 * q + s - 1;
            if (h < 0 || h >= H || w < 0 || w >= W) continue;  // padding never wins
            float4 v4 = tap[r * 3 + s];
            if (INAFF)  // the BN + ReLU output as the normalising kernel would have stored it
                v4 = as_stored(y, make_float4(fmaxf(fmaf(v4.x, sc.x, sh.x), 0.f), fmaxf(fmaf(v4.y, sc.y, sh.y), 0.f),
                                              fmaxf(fmaf(v4.z, sc.z, sh.z), 0.f), fmaxf(fmaf(v4.w, sc.w, sh.w), 0.f)));
            const float v[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (bi[e] < 0 || v[e] > best[e]) {  // strict: the first maximal element in window order wins
                    best[e] = v[e];
                    bi[e] = r * 3 + s;
                }
        }
    st4(y, i, make_float4(best[0], best[1], best[2], best[3]));
    reinterpret_cast<uchar4 *>(arg)[i] = make_uchar4((uint8_t)bi[0], (uint8_t)bi[1], (uint8_t)bi[2], (uint8_t)bi[3]);
}

// Gather form: a pixel sums the windows that elected it.  One thread per (n, 2x2 block of pixels, 4 channels): pixel
// (2b + dh, 2a + dw) lies in windows p in {b, b + dh}, q in {a, a + dw}, so the block's four pixels share four windows,
// loaded once (one thread per pixel loads each window up to four times and is bound by the load units, not by memory).
// Each pixel adds its windows in (p, q) order.
template <class T, bool DY2>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(int N, int C4, int H, int W, int P, int Q, const T *__restrict__ dy,
                                                          const T *__restrict__ dy2, const uint8_t *__restrict__ arg,
                                                          T *__restrict__ dx)
{
    const int HB = (H + 1) / 2, WB = (W + 1) / 2;
    // neighbouring blocks share windows: keep them on one XCD
    const size_t i = (size_t)xcd_contiguous(blockIdx.x, gridDim.x) * 256 + threadIdx.x;
    if (i >= (size_t)N * HB * WB * C4) return;
    const unsigned iu = (unsigned)i;  // 32-bit index arithmetic (the host checks the element count)
    const int c = (int)(iu % (unsigned)C4);
    unsigned t = iu / (unsigned)C4;
    const int wb = (int)(t % (unsigned)WB);
    t /= (unsigned)WB;
    const int hb = (int)(t % (unsigned)HB), n = (int)(t / (unsigned)HB);
    // the four windows (hb + i, wb + j), loaded at clamped positions so that all loads are in flight together
    uchar4 a[4];
    float4 g[4];
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) {
        const int p = min(hb + (t4 >> 1), P - 1), q = min(wb + (t4 & 1), Q - 1);
        const size_t o = ((size_t)(n * P + p) * Q + q) * C4 + c;
        a[t4] = reinterpret_cast<const uchar4 *>(arg)[o];
        g[t4] = ld4(dy, o);
        if (DY2) {
            const float4 g2 = ld4(dy2, o);
            g[t4].x += g2.x; g[t4].y += g2.y; g[t4].z += g2.z; g[t4].w += g2.w;
        }
    }
#pragma unroll
    for (int dh = 0; dh < 2; ++dh)
#pragma unroll
        for (int dw = 0; dw < 2; ++dw) {
            const int h = 2 * hb + dh, w = 2 * wb + dw;
            if (h >= H || w >= W) continue;
            float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t4 = 0; t4 < 4; ++t4) {
                const int ip = t4 >> 1, iq = t4 & 1;
                if (ip > dh || iq > dw || hb + ip >= P || wb + iq >= Q) continue;  // not a window of this pixel
                const int want = (h - (2 * (hb + ip) - 1)) * 3 + (w - (2 * (wb + iq) - 1));
                if (a[t4].x == want) acc[0] += g[t4].x;
                if (a[t4].y == want) acc[1] += g[t4].y;
                if (a[t4].z == want) acc[2] += g[t4].z;
                if (a[t4].w == want) acc[3] += g[t4].w;
            }
            st4(dx, ((size_t)(n * H + h) * W + w) * C4 + c, make_float4(acc[0], acc[1], acc[2], acc[3]));
        }
}

// Workgroup = 64 float4 columns x 4 slices of the H*W positions; the four slice sums are added in slice order.
template <class T>
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(int N, int C4, int HW, const T *__restrict__ x, float *__restrict__ y)
{
    __shared__ float4 red[4][64];
    const int cl = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + cl, n = blockIdx.y;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < C4)
        for (int j = slice; j < HW; j += 4) {
            const float4 v = ld4(x, ((size_t)n * HW + j) * C4 + c);
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
    red[slice][cl] = s;
    __syncthreads();
    if (slice == 0 && c < C4) {
        for (int t = 1; t < 4; ++t) {
            const float4 v = red[t][cl];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        const float inv = 1.0f / (float)HW;
        reinterpret_cast<float4 *>(y)[(size_t)n * C4 + c] = make_float4(s.x * inv, s.y * inv, s.z * inv, s.w * inv);
    }
}

template <class T>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(int N, int C4, int HW, const float *__restrict__ dy, T *__restrict__ dx)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)N * HW * C4) return;
    const unsigned iu = (unsigned)i;  // 32-bit index arithmetic (the host checks the element count)
    const int c = (int)(iu % (unsigned)C4);
    const int n = (int)(iu / ((unsigned)HW * (unsigned)C4));
    const float4 g = ld4(dy, (size_t)n * C4 + c);
    const float inv = 1.0f / (float)HW;
    st4(dx, i, make_float4(g.x * inv, g.y * inv, g.z * inv, g.w * inv));
}

// y[n,k] = <f[n,:], w[k,:]> + b[k]: one workgroup per output class and tile of up to 32 samples; its four wavefronts
// take interleaved quarters of the reduction and their partial sums are added in wavefront order through LDS.
// (Four classes per workgroup, so that a feature load serves four of them, measured slower: 28 -> 42 us.)
constexpr int kFcTileN = 32;
__global__ __launch_bounds__(256) void fc_fwd_kernel(int N, int J, int K, const float *__restrict__ f, const float *__restrict__ w,
                                                     const float *__restrict__ b, float *__restrict__ y)
{
    __shared__ float part[4][kFcTileN];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = blockIdx.x;
    const int n0 = blockIdx.y * kFcTileN;
    float acc[kFcTileN];
#pragma unroll
    for (int n = 0; n < kFcTileN; ++n) acc[n] = 0.f;
    for (int j = (wave * 64 + lane) * 4; j < J; j += 1024) {
        const float4 wv = *reinterpret_cast<const float4 *>(w + (size_t)k * J + j);
        // sixteen feature loads in flight at a time (a load used right away costs a round trip each); rows past the batch
        // repeat the last sample and are never stored
#pragma unroll
        for (int nb = 0; nb < kFcTileN; nb += 16) {
            float4 fv[16];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                fv[u] = *reinterpret_cast<const float4 *>(f + (size_t)min(n0 + nb + u, N - 1) * J + j);
#pragma unroll
            for (int u = 0; u < 16; ++u)
                acc[nb + u] = fmaf(fv[u].x, wv.x, fmaf(fv[u].y, wv.y, fmaf(fv[u].z, wv.z, fmaf(fv[u].w, wv.w, acc[nb + u]))));
        }
    }
#pragma unroll
    for (int n = 0; n < kFcTileN; ++n) {
        const float s = wave_sum(acc[n]);
        if (lane == 0) part[wave][n] = s;
    }
    __syncthreads();
    const int n = threadIdx.x;
    if (n < kFcTileN && n0 + n < N) y[(size_t)(n0 + n) * K + k] = ((part[0][n] + part[1][n]) + (part[2][n] + part[3][n])) + b[k];
}

// dw[k,j] = sum_n dy[n,k] f[n,j]; db[k] = sum_n dy[n,k].  One thread per (k, 4 columns).
__global__ __launch_bounds__(256) void fc_bwd_weight_kernel(int N, int J4, int K, const float *__restrict__ f,
                                                            const float *__restrict__ dy, float *__restrict__ dw, float *__restrict__ db)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (size_t)K * J4) return;
    const int k = (int)(i / J4), j = (int)(i - (size_t)k * J4);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float sb = 0.f;
    int n = 0;
    for (; n + 7 < N; n += 8) {  // eight samples' loads in flight, added in sample order
        float g[8];
        float4 fv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            g[u] = dy[(size_t)(n + u) * K + k];
            fv[u] = ld4(f, (size_t)(n + u) * J4 + j);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc.x = fmaf(g[u], fv[u].x, acc.x); acc.y = fmaf(g[u], fv[u].y, acc.y);
            acc.z = fmaf(g[u], fv[u].z, acc.z); acc.w = fmaf(g[u], fv[u].w, acc.w);
            sb += g[u];
        }
    }
    for (; n < N; ++n) {
        const float g = dy[(size_t)n * K + k];
        const float4 fv = ld4(f, (size_t)n * J4 + j);
        acc.x = fmaf(g, fv.x, acc.x); acc.y = fmaf(g, fv.y, acc.y); acc.z = fmaf(g, fv.z, acc.z); acc.w = fmaf(g, fv.w, acc.w);
        sb += g;
    }
    reinterpret_cast<float4 *>(dw)[i] = acc;
    if (j == 0) db[k] = sb;
}

// df[n,j] = sum_k dy[n,k] w[k,j].  Workgroup = 64 float4 columns x 16 slices of k, eight loads in flight per thread; the
// slice sums are added in slice order through LDS (a fixed order).
constexpr int kFcSlices = 16;
__global__ __launch_bounds__(64 * kFcSlices) void fc_bwd_data_kernel(int N, int J4, int K, const float *__restrict__ w,
                                                                    const float *__restrict__ dy, float *__restrict__ df)
{
    __shared__ float4 red[kFcSlices][64];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63);
    const int slice = threadIdx.x >> 6;
    const int n = blockIdx.y;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (col < J4) {
        const int per = (K + kFcSlices - 1) / kFcSlices;
        const int kb = per * slice, ke = min(K, kb + per);
#pragma unroll 8
        for (int k = kb; k < ke; ++k) {
            const float g = dy[(size_t)n * K + k];
            const float4 wv = ld4(w, (size_t)k * J4 + col);
            acc.x = fmaf(g, wv.x, acc.x); acc.y = fmaf(g, wv.y, acc.y); acc.z = fmaf(g, wv.z, acc.z); acc.w = fmaf(g, wv.w, acc.w);
        }
    }
    red[slice][threadIdx.x & 63] = acc;
    __syncthreads();
    if (slice == 0 && col < J4) {
        float4 s = red[0][threadIdx.x];
        for (int t = 1; t < kFcSlices; ++t) {
            const float4 v = red[t][threadIdx.x];
            s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
        }
        reinterpret_cast<float4 *>(df)[(size_t)n * J4 + col] = s;
    }
}

// Single workgroup of 16 wavefronts; each wavefront takes rows wave, wave+16, ...  Row losses are summed in row order.
constexpr int kSoftmaxRegs = 16;  // rows of up to 1024 classes are held in registers
__global__ __launch_bounds__(1024) void softmax_ce_kernel(int N, int K, const float *__restrict__ logits, const int32_t *__restrict__ labels,
                                                          float *__restrict__ loss, float *__restrict__ dlogits)
{
    __shared__ float row_loss[1024];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float invN = 1.0f / (float)N;
    for (int n = wave; n < N; n += 16) {
        const float *z = logits + (size_t)n * K;
        const int lab = labels[n];
        // a label outside [0, K) makes the loss NaN (and puts no one-hot term into the gradient); z[lab] is never read for it
        const bool lab_ok = (unsigned)lab < (unsigned)K;
        if (K <= 64 * kSoftmaxRegs) {
            // the row fits in registers: one round of loads in flight instead of three dependent passes over memory
            float v[kSoftmaxRegs];
#pragma unroll
            for (int i = 0; i < kSoftmaxRegs; ++i) v[i] = lane + 64 * i < K ? z[lane + 64 * i] : -INFINITY;
            float mx = v[0];
#pragma unroll
            for (int i = 1; i < kSoftmaxRegs; ++i) mx = fmaxf(mx, v[i]);
            mx = wave_max(mx);
            float se = 0.f;
#pragma unroll
            for (int i = 0; i < kSoftmaxRegs; ++i) se += lane + 64 * i < K ? expf(v[i] - mx) : 0.f;
            se = wave_sum(se);
            const float lse = mx + logf(se);
#pragma unroll
            for (int i = 0; i < kSoftmaxRegs; ++i) {
                const int k = lane + 64 * i;
                if (k < K) dlogits[(size_t)n * K + k] = (expf(v[i] - lse) - (k == lab ? 1.f : 0.f)) * invN;
            }
            if (lane == 0) row_loss[n] = lab_ok ? lse - z[lab] : __builtin_nanf("");
            continue;
        }
        float mx = -INFINITY;
        for (int k = lane; k < K; k += 64) mx = fmaxf(mx, z[k]);
        mx = wave_max(mx);
        float se = 0.f;
        for (int k = lane; k < K; k += 64) se += expf(z[k] - mx);
        se = wave_sum(se);
        const float lse = mx + logf(se);
        for (int k = lane; k < K; k += 64) dlogits[(size_t)n * K + k] = (expf(z[k] - lse) - (k == lab ? 1.f : 0.f)) * invN;
        if (lane == 0) row_loss[n] = lab_ok ? lse - z[lab] : __builtin_nanf("");
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float s = 0.f;
        for (int n = 0; n < N; ++n) s += row_loss[n];
        loss[0] = s * invN;
    }
}

static int dims_check(const char *who, int n, int c, int h, int w)
{
    RN50_REQUIRE(n > 0 && c > 0 && h > 0 && w > 0, RN50_EINVAL, "%s: non-positive dimension", who);
    RN50_REQUIRE(c % 4 == 0, RN50_EUNSUPPORTED, "%s: channel count must be a multiple of 4", who);
    RN50_REQUIRE((long)n * h * w * c < (1L << 31), RN50_EUNSUPPORTED, "%s: tensor too large", who);
    return RN50_OK;
}

}  // namespace rn50

using namespace rn50;

template <class T>
static int maxpool_fwd_impl(const char *who, int n, int c, int h, int w, const T *x, const float *in_scale, const float *in_shift,
                            T *y, uint8_t *argidx, void *stream)
{
    if (int rc = dims_check(who, n, c, h, w)) return rc;
    RN50_REQUIRE(x && y && argidx, RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(x) && aligned16(y) && aligned16(argidx) && aligned16(in_scale) && aligned16(in_shift), RN50_EINVAL,
                 "%s: pointers must be 16-byte aligned", who);
    RN50_REQUIRE((in_scale != nullptr) == (in_shift != nullptr), RN50_EINVAL, "%s: scale and shift go together", who);
    const int P = (h - 1) / 2 + 1, Q = (w - 1) / 2 + 1;
    const size_t total = (size_t)n * P * Q * (c / 4);
    RN50_REQUIRE((size_t)n * h * w * (c / 4) < (1ull << 31), RN50_EUNSUPPORTED, "%s: more than 2^31 groups of four channels", who);
    if (in_scale)
        hipLaunchKernelGGL((maxpool_fwd_kernel<T, true>), dim3(ceil_div(total, 256)), dim3(256), 0, (hipStream_t)stream, n, c / 4, h, w, P, Q, x,
                           in_scale, in_shift, y, argidx);
    else
        hipLaunchKernelGGL((maxpool_fwd_kernel<T, false>), dim3(ceil_div(total, 256)), dim3(256), 0, (hipStream_t)stream, n, c / 4, h, w, P, Q, x,
                           in_scale, in_shift, y, argidx);
    return launch_status(who);
}

extern "C" int maxpool3x3s2_fwd(int n, int c, int h, int w, const float *x, float *y, uint8_t *argidx, void *stream)
{
    return maxpool_fwd_impl<float>("maxpool3x3s2_fwd", n, c, h, w, x, nullptr, nullptr, y, argidx, stream);
}

extern "C" int maxpool3x3s2_fwd_bnrelu_input(int n, int c, int h, int w, const float *x, const float *in_scale, const float *in_shift,
                                             float *y, uint8_t *argidx, void *stream)
{
    RN50_REQUIRE(in_scale && in_shift, RN50_EINVAL, "maxpool3x3s2_fwd_bnrelu_input: null scale or shift");
    return maxpool_fwd_impl<float>("maxpool3x3s2_fwd_bnrelu_input", n, c, h, w, x, in_scale, in_shift, y, argidx, stream);
}

extern "C" int maxpool3x3s2_fwd_bf16(int n, int c, int h, int w, const uint16_t *x, const float *in_scale_or_null,
                                     const float *in_shift_or_null, uint16_t *y, uint8_t *argidx, void *stream)
{
    return maxpool_fwd_impl<bf16_t>("maxpool3x3s2_fwd_bf16", n, c, h, w, x, in_scale_or_null, in_shift_or_null, y, argidx, stream);
}

template <class T>
static int maxpool_bwd_impl(const char *who, int n, int c, int h, int w, const T *dy, const T *dy2_or_null, const uint8_t *argidx, T *dx,
                            void *stream)
{
    if (int rc = dims_check(who, n, c, h, w)) return rc;
    RN50_REQUIRE(dy && dx && argidx, RN50_EINVAL, "%s: null pointer", who);
    RN50_REQUIRE(aligned16(dy) && aligned16(dy2_or_null) && aligned16(dx) && aligned16(argidx), RN50_EINVAL,
                 "%s: pointers must be 16-byte aligned", who);
    const int P = (h - 1) / 2 + 1, Q = (w - 1) / 2 + 1;
    RN50_REQUIRE((size_t)n * h * w * (c / 4) < (1ull << 31), RN50_EUNSUPPORTED, "%s: more than 2^31 groups of four channels", who);
    const size_t total = (size_t)n * ((h + 1) / 2) * ((w + 1) / 2) * (c / 4);  // one thread per 2x2 block of pixels
    if (dy2_or_null)
        hipLaunchKernelGGL((maxpool_bwd_kernel<T, true>), dim3(ceil_div(total, 256)), dim3(256), 0, (hipStream_t)stream, n, c / 4, h, w, P, Q, dy,
                           dy2_or_null, argidx, dx);
    else
        hipLaunchKernelGGL((maxpool_bwd_kernel<T, false>), dim3(ceil_div(total, 256)), dim3(256), 0, (hipStream_t)stream, n, c / 4, h, w, P, Q, dy,
                           dy2_or_null, argidx, dx);
    return launch_status(who);
}

extern "C" int maxpool3x3s2_bwd(int n, int c, int h, int w, const float *dy, const float *dy2_or_null, const uint8_t *argidx,
                                float *dx, void *stream)
{
    return maxpool_bwd_impl<float>("maxpool3x3s2_bwd", n, c, h, w, dy, dy2_or_null, argidx, dx, stream);
}

extern "C" int maxpool3x3s2_bwd_bf16(int n, int c, int h, int w, const uint16_t *dy, const uint16_t *dy2_or_null, const uint8_t *argidx,
                                     uint16_t *dx, void *stream)
{
    return maxpool_bwd_impl<bf16_t>("maxpool3x3s2_bwd_bf16", n, c, h, w, dy, dy2_or_null, argidx, dx, stream);
}

template <class T>
static int avgpool_fwd_impl(const char *who, int n, int c, int h, int w, const T *x, float *y, void *stream)
{
    if (int rc = dims_check(who, n, c, h, w)) return rc;
    RN50_REQUIRE(x && y && aligned16(x) && aligned16(y), RN50_EINVAL, "%s: null or misaligned pointer", who);
    hipLaunchKernelGGL((avgpool_fwd_kernel<T>), dim3(ceil_div(c / 4, 64), n), dim3(256), 0, (hipStream_t)stream, n, c / 4, h * w, x, y);
    return launch_status(who);
}

template <class T>
static int avgpool_bwd_impl(const char *who, int n, int c, int h, int w, const float *dy, T *dx, void *stream)
{
    if (int rc = dims_check(who, n, c, h, w)) return rc;
    RN50_REQUIRE(dy && dx && aligned16(dy) && aligned16(dx), RN50_EINVAL, "%s: null or misaligned pointer", who);
    RN50_REQUIRE((size_t)n * h * w * (c / 4) < (1ull << 31), RN50_EUNSUPPORTED, "%s: more than 2^31 groups of four channels", who);
    hipLaunchKernelGGL((avgpool_bwd_kernel<T>), dim3(ceil_div((long)n * h * w * c / 4, 256)), dim3(256), 0, (hipStream_t)stream, n, c / 4, h * w, dy, dx);
    return launch_status(who);
}

extern "C" int avgpool_fwd(int n, int c, int h, int w, const float *x, float *y, void *stream)
{
    return avgpool_fwd_impl<float>("avgpool_fwd", n, c, h, w, x, y, stream);
}
extern "C" int avgpool_bwd(int n, int c, int h, int w, const float *dy, float *dx, void *stream)
{
    return avgpool_bwd_impl<float>("avgpool_bwd", n, c, h, w, dy, dx, stream);
}
extern "C" int avgpool_fwd_bf16(int n, int c, int h, int w, const uint16_t *x, float *y, void *stream)
{
    return avgpool_fwd_impl<bf16_t>("avgpool_fwd_bf16", n, c, h, w, x, y, stream);
}
extern "C" int avgpool_bwd_bf16(int n, int c, int h, int w, const float *dy, uint16_t *dx, void *stream)
{
    return avgpool_bwd_impl<bf16_t>("avgpool_bwd_bf16", n, c, h, w, dy, dx, stream);
}

extern "C" int fc_fwd(int n, int j, int k, const float *f, const float *w, const float *b, float *y, void *stream)
{
    RN50_REQUIRE(n > 0 && j > 0 && k > 0, RN50_EINVAL, "fc_fwd: non-positive dimension");
    RN50_REQUIRE(j % 4 == 0, RN50_EUNSUPPORTED, "fc_fwd: input width must be a multiple of 4");
    RN50_REQUIRE(f && w && b && y && aligned16(f) && aligned16(w) && aligned16(b) && aligned16(y), RN50_EINVAL,
                 "fc_fwd: null or misaligned pointer");
    hipLaunchKernelGGL(fc_fwd_kernel, dim3(k, ceil_div(n, kFcTileN)), dim3(256), 0, (hipStream_t)stream, n, j, k, f, w, b, y);
    return launch_status("fc_fwd");
}

extern "C" int fc_bwd(int n, int j, int k, const float *f, const float *w, const float *dy, float *df, float *dw, float *db,
                      void *stream)
{
    RN50_REQUIRE(n > 0 && j > 0 && k > 0, RN50_EINVAL, "fc_bwd: non-positive dimension");
    RN50_REQUIRE(j % 4 == 0, RN50_EUNSUPPORTED, "fc_bwd: input width must be a multiple of 4");
    RN50_REQUIRE(f && w && dy && df && dw && db, RN50_EINVAL, "fc_bwd: null pointer");
    RN50_REQUIRE(aligned16(f) && aligned16(w) && aligned16(dy) && aligned16(df) && aligned16(dw) && aligned16(db), RN50_EINVAL,
                 "fc_bwd: pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(fc_bwd_weight_kernel, dim3(ceil_div((long)k * j / 4, 256)), dim3(256), 0, st, n, j / 4, k, f, dy, dw, db);
    hipLaunchKernelGGL(fc_bwd_data_kernel, dim3(ceil_div(j / 4, 64), n), dim3(64 * kFcSlices), 0, st, n, j / 4, k, w, dy, df);
    return launch_status("fc_bwd");
}

extern "C" int softmax_ce(int n, int k, const float *logits, const int32_t *labels, float *loss, float *dlogits, void *stream)
{
    RN50_REQUIRE(n > 0 && k > 0, RN50_EINVAL, "softmax_ce: non-positive dimension");
    RN50_REQUIRE(n <= 1024, RN50_EUNSUPPORTED, "softmax_ce: at most 1024 rows");
    RN50_REQUIRE(logits && labels && loss && dlogits, RN50_EINVAL, "softmax_ce: null pointer");
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(1), dim3(1024), 0, (hipStream_t)stream, n, k, logits, labels, loss, dlogits);
    return launch_status("softmax_ce");
}
